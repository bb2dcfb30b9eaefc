"""Python binding of libdessert_hip.so (the C ABI declared in include/dessert.h).

Argument marshalling only: torch supplies device memory and the HIP stream,
every step of hashing, scoring and top-k runs in the library's gfx950 kernels.
There is no CPU path: loading fails loudly if the shared library has not been
built (run ``python -m paper_2210_15748_amd.build`` or ``__graft_entry__.build()``).

Function names mirror the C entry points without the ``dessert_`` prefix:
``create`` / ``destroy`` / ``hash`` / ``build_index`` / ``search`` / ``scores`` /
``set_algo`` / ``set_score_transform`` / ``get_projection`` / ``enable_timing`` / ``get_timing``.
"""
from __future__ import annotations

import ctypes as C
import os
import pathlib
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = pathlib.Path(__file__).resolve().parent
LIB_PATH = _HERE / "libdessert_hip.so"

OK, EINVAL, ENOMEM, EHIP, ESTATE = range(5)
I8, F16 = 0, 1
PROJ_RADEMACHER_I8, PROJ_GAUSSIAN_F32 = 0, 1
HASH_AUTO, HASH_SCALAR, HASH_MFMA = 0, 1, 2
SCORE_AUTO, SCORE_BYTECMP, SCORE_MASKLUT = 0, 1, 2

SCORE_RAW_COUNTS, SCORE_EQ1_Q16 = 0, 1
SCORE_MAX_IDENTITY_Q16, SCORE_MAX_EXPM1_Q16, SCORE_MAX_SIGMOID_Q16 = 2, 3, 4
SCORE_MEAN_IDENTITY_Q16, SCORE_MEAN_EXPM1_Q16, SCORE_MEAN_SIGMOID_Q16 = 5, 6, 7

EXPORTS = [
    "dessert_create", "dessert_destroy", "dessert_get_projection", "dessert_set_algo", "dessert_set_score_transform",
    "dessert_set_query_weights",
    "dessert_code_bytes",
    "dessert_hash", "dessert_build_index", "dessert_attach_index", "dessert_search_workspace_bytes", "dessert_search", "dessert_scores",
    "dessert_noalloc_scratch_bytes", "dessert_search_noalloc", "dessert_set_debug", "dessert_last_score_kernel",
    "dessert_filter_kmeans_workspace_bytes", "dessert_filter_kmeans",
    "dessert_filter_build", "dessert_filter_workspace_bytes", "dessert_filter_query",
    "dessert_filter_search_workspace_bytes", "dessert_filter_search",
    "dessert_enable_timing", "dessert_get_timing", "dessert_probe_read_bandwidth", "dessert_probe_mix_bandwidth", "dessert_last_error",
    "dessert_version",
]


class Config(C.Structure):
    _fields_ = [("d", C.c_uint32), ("L", C.c_uint32), ("C", C.c_uint32), ("dtype", C.c_uint32),
                ("proj_kind", C.c_uint32), ("device", C.c_int32), ("seed", C.c_uint64),
                ("proj_dev", C.c_void_p), ("stream", C.c_void_p)]


class DessertError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"dessert status {status}: {message}")
        self.status = status


_lib = None


def lib() -> C.CDLL:
    """Load the shared library (once) and declare its signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not LIB_PATH.exists():
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2210_15748_amd.build`; "
                          "there is no fallback implementation")
    l = C.CDLL(os.fspath(LIB_PATH))
    vp, u32, u64, sz = C.c_void_p, C.c_uint32, C.c_uint64, C.c_size_t
    l.dessert_create.argtypes = [C.POINTER(Config), C.POINTER(vp)]
    l.dessert_destroy.argtypes = [vp]
    l.dessert_destroy.restype = None
    l.dessert_get_projection.argtypes = [vp, vp]
    l.dessert_set_algo.argtypes = [vp, C.c_int, C.c_int]
    l.dessert_set_score_transform.argtypes = [vp, C.c_int]
    l.dessert_set_query_weights.argtypes = [vp, vp, u64]
    l.dessert_code_bytes.argtypes = [vp, u64]
    l.dessert_code_bytes.restype = sz
    l.dessert_hash.argtypes = [vp, vp, u64, vp]
    l.dessert_build_index.argtypes = [vp, vp, u64, vp, u64, vp, vp]
    l.dessert_attach_index.argtypes = [vp, vp, vp, u64, u64, u64]
    l.dessert_search_workspace_bytes.argtypes = [vp, u32, u64, u64, u32]
    l.dessert_search_workspace_bytes.restype = sz
    l.dessert_search.argtypes = [vp, vp, vp, u32, vp, vp, u32, vp, sz, vp, vp]
    l.dessert_scores.argtypes = [vp, vp, vp, u32, vp, vp, vp, sz, vp]
    l.dessert_noalloc_scratch_bytes.argtypes = []
    l.dessert_noalloc_scratch_bytes.restype = sz
    l.dessert_search_noalloc.argtypes = [vp, vp, u32, u32, vp, u64, u32, vp, vp]
    l.dessert_set_debug.argtypes = [vp, C.c_int]
    l.dessert_last_score_kernel.argtypes = [vp]
    l.dessert_last_score_kernel.restype = C.c_char_p
    l.dessert_filter_kmeans_workspace_bytes.argtypes = [vp, u64, u32]
    l.dessert_filter_kmeans_workspace_bytes.restype = sz
    l.dessert_filter_kmeans.argtypes = [vp, vp, u64, vp, u32, u32, vp, sz]
    l.dessert_filter_build.argtypes = [vp, vp, u32, vp, vp, vp, vp]
    l.dessert_filter_workspace_bytes.argtypes = [vp, u32, u64, u32, u32]
    l.dessert_filter_workspace_bytes.restype = sz
    l.dessert_filter_query.argtypes = [vp, vp, vp, u32, u32, u32, vp, sz, vp, vp]
    l.dessert_filter_search_workspace_bytes.argtypes = [vp, u32, u64, u32, u32, u32, u32]
    l.dessert_filter_search_workspace_bytes.restype = sz
    l.dessert_filter_search.argtypes = [vp, vp, vp, u32, u32, u32, u32, vp, sz, vp, vp]
    l.dessert_enable_timing.argtypes = [vp, C.c_int]
    l.dessert_get_timing.argtypes = [vp, u32, C.POINTER(C.c_float)]
    l.dessert_probe_read_bandwidth.argtypes = [vp, sz, C.c_int, vp, C.c_int, C.POINTER(C.c_float)]
    l.dessert_probe_mix_bandwidth.argtypes = [vp, vp, sz, C.c_int, vp, C.c_int, C.POINTER(C.c_float)]
    l.dessert_last_error.restype = C.c_char_p
    l.dessert_version.restype = C.c_char_p
    _lib = l
    return l


def last_error() -> str:
    return lib().dessert_last_error().decode()


def version() -> str:
    return lib().dessert_version().decode()


def _check(status: int):
    if status != OK:
        raise DessertError(status, last_error())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _host_u32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a.cpu() if isinstance(a, torch.Tensor) else a), dtype=np.uint32)


def _host_u64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a.cpu() if isinstance(a, torch.Tensor) else a), dtype=np.uint64)


class Index:
    """Owner of one dessert_index_t handle plus the torch buffers the index lives in."""

    def __init__(self, handle: int, cfg: Config, device: torch.device):
        self.handle = handle
        self.cfg = cfg
        self.device = device
        self.codes: Optional[torch.Tensor] = None
        self.offsets: Optional[torch.Tensor] = None
        self.n_docs = 0
        self._keep = []

    def __del__(self):
        try:
            destroy(self)
        except Exception:
            pass


def create(d: int, L: int, C_bits: int, dtype: int = I8, proj_kind: int = PROJ_RADEMACHER_I8,
           proj: Optional[torch.Tensor] = None, seed: int = 0, device: Optional[torch.device] = None,
           stream: Optional[torch.cuda.Stream] = None) -> Index:
    """dessert_create.  ``proj``: device tensor [L*C, d] (int8 or float32) or None (seed-derived)."""
    if device is None:
        device = proj.device if proj is not None else torch.device("cuda", torch.cuda.current_device())
    device = torch.device(device)
    dev_index = device.index if device.index is not None else torch.cuda.current_device()
    if stream is None:
        stream = torch.cuda.current_stream(device)
    cfg = Config(d=d, L=L, C=C_bits, dtype=dtype, proj_kind=proj_kind, device=dev_index, seed=seed,
                 proj_dev=_ptr(proj.contiguous() if proj is not None else None), stream=stream.cuda_stream)
    if proj is not None:
        want = torch.int8 if proj_kind == PROJ_RADEMACHER_I8 else torch.float32
        if proj.dtype != want or tuple(proj.shape) != (L * C_bits, d) or not proj.is_cuda:
            raise ValueError("proj must be a device tensor [L*C, d] of dtype " + str(want))
    handle = C.c_void_p()
    _check(lib().dessert_create(C.byref(cfg), C.byref(handle)))
    return Index(handle.value, cfg, torch.device("cuda", dev_index))


def destroy(ix: Index) -> None:
    if ix.handle:
        lib().dessert_destroy(ix.handle)
        ix.handle = None


def set_algo(ix: Index, hash_algo: int = HASH_AUTO, score_algo: int = SCORE_AUTO) -> None:
    _check(lib().dessert_set_algo(ix.handle, hash_algo, score_algo))


def set_score_transform(ix: Index, transform: int) -> None:
    _check(lib().dessert_set_score_transform(ix.handle, transform))


def set_query_weights(ix: Index, weights: Optional[torch.Tensor]) -> None:
    """dessert_set_query_weights: a device tensor of Q16 weights (uint32 / int32 values in 0..65536), one per query
    vector of the following batches, or None."""
    if weights is None:
        ix._weights = None
        _check(lib().dessert_set_query_weights(ix.handle, None, 0))
        return
    if not weights.is_cuda or weights.dtype not in (torch.int32, torch.uint32) or weights.dim() != 1:
        raise ValueError("weights must be a 1-d device tensor of int32 / uint32")
    ix._weights = weights.contiguous()
    _check(lib().dessert_set_query_weights(ix.handle, ix._weights.data_ptr(), ix._weights.numel()))


def get_projection(ix: Index) -> torch.Tensor:
    dt = torch.int8 if ix.cfg.proj_kind == PROJ_RADEMACHER_I8 else torch.float32
    out = torch.empty(ix.cfg.L * ix.cfg.C, ix.cfg.d, dtype=dt, device=ix.device)
    _check(lib().dessert_get_projection(ix.handle, out.data_ptr()))
    return out


def _check_vectors(ix: Index, v: torch.Tensor) -> torch.Tensor:
    want = torch.int8 if ix.cfg.dtype == I8 else torch.float16
    if not v.is_cuda or v.dtype != want or v.dim() != 2 or v.shape[1] != ix.cfg.d:
        raise ValueError(f"vectors must be a device tensor [n, {ix.cfg.d}] of dtype {want}")
    return v.contiguous()


def code_dtype(ix: Index) -> torch.dtype:
    """Element type of the code arrays: uint8, or uint16 when C > 8."""
    return torch.uint16 if ix.cfg.C > 8 else torch.uint8


def hash(ix: Index, vectors: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:  # noqa: A001
    """dessert_hash: codes [n, L] of code_dtype(ix)."""
    vectors = _check_vectors(ix, vectors)
    n = vectors.shape[0]
    if out is None:
        out = torch.empty(n, ix.cfg.L, dtype=code_dtype(ix), device=ix.device)
    _check(lib().dessert_hash(ix.handle, vectors.data_ptr(), n, out.data_ptr()))
    return out


def build_index(ix: Index, vectors: torch.Tensor, lengths, codes: Optional[torch.Tensor] = None,
                offsets: Optional[torch.Tensor] = None):
    """dessert_build_index.  Returns (codes [V, L] of code_dtype(ix), offsets [N+1] int64), both on the device."""
    vectors = _check_vectors(ix, vectors)
    lens = _host_u32(lengths)
    n_docs, V = lens.shape[0], vectors.shape[0]
    if codes is None:
        codes = torch.empty(V, ix.cfg.L, dtype=code_dtype(ix), device=ix.device)
    if offsets is None:
        offsets = torch.empty(n_docs + 1, dtype=torch.int64, device=ix.device)
    _check(lib().dessert_build_index(ix.handle, vectors.data_ptr(), V, lens.ctypes.data, n_docs,
                                     codes.data_ptr(), offsets.data_ptr()))
    ix.codes, ix.offsets, ix.n_docs = codes, offsets, n_docs
    return codes, offsets


def attach_index(ix: Index, codes: torch.Tensor, offsets: torch.Tensor, max_length: Optional[int] = None) -> None:
    """dessert_attach_index: make arrays written by an earlier build_index (same configuration and projection matrix) this
    handle's index.  max_length (longest document) is computed from the offsets if not given."""
    if not codes.is_cuda or not offsets.is_cuda or offsets.dtype != torch.int64 or offsets.dim() != 1 or offsets.numel() < 1:
        raise ValueError("codes and offsets must be device tensors, offsets int64 [n_docs + 1]")
    if codes.dtype != code_dtype(ix) or codes.dim() != 2 or codes.shape[1] != ix.cfg.L:
        raise ValueError(f"codes must be [n_vectors, {ix.cfg.L}] of {code_dtype(ix)}")
    codes, offsets = codes.contiguous(), offsets.contiguous()
    n_docs = offsets.numel() - 1
    if max_length is None:
        max_length = int((offsets[1:] - offsets[:-1]).max().item()) if n_docs else 0
    _check(lib().dessert_attach_index(ix.handle, codes.data_ptr(), offsets.data_ptr(), n_docs, codes.shape[0], max_length))
    ix.codes, ix.offsets, ix.n_docs = codes, offsets, n_docs


def _batch(ix: Index, q_vectors, q_lengths, cand_ids, cand_offsets):
    q_vectors = _check_vectors(ix, q_vectors)
    ql = _host_u32(q_lengths)
    B = ql.shape[0]
    if int(ql.sum()) != q_vectors.shape[0]:
        raise ValueError("sum(q_lengths) != number of query vectors")
    if cand_ids is not None:
        if cand_ids.dim() == 2 and cand_offsets is None:
            cand_offsets = np.arange(B + 1, dtype=np.uint64) * cand_ids.shape[1]
        if cand_ids.dtype != torch.int32 and cand_ids.dtype != torch.uint32:
            cand_ids = cand_ids.to(torch.int32)
        cand_ids = cand_ids.contiguous().reshape(-1)
        co = _host_u64(cand_offsets)
        if co.shape[0] != B + 1 or int(co[-1]) != cand_ids.numel():
            raise ValueError("cand_offsets must have n_queries+1 entries ending at len(cand_ids)")
        total = int(co[-1])
    else:
        co = None
        total = B * ix.n_docs
    return q_vectors, ql, B, cand_ids, co, total


def workspace_bytes(ix: Index, n_queries: int, total_q_vectors: int, total_scored: int, k: int) -> int:
    return int(lib().dessert_search_workspace_bytes(ix.handle, n_queries, total_q_vectors, total_scored, k))


def search(ix: Index, q_vectors: torch.Tensor, q_lengths, k: int, cand_ids: Optional[torch.Tensor] = None,
           cand_offsets=None, workspace: Optional[torch.Tensor] = None, out_ids: Optional[torch.Tensor] = None,
           out_scores: Optional[torch.Tensor] = None):
    """dessert_search.  Returns (ids [B, k] int64 view of uint32, scores [B, k] int32)."""
    q_vectors, ql, B, cand_ids, co, total = _batch(ix, q_vectors, q_lengths, cand_ids, cand_offsets)
    if workspace is None:
        workspace = torch.empty(workspace_bytes(ix, B, q_vectors.shape[0], total, k), dtype=torch.uint8,
                                device=ix.device)
    if out_ids is None:
        out_ids = torch.empty(B, k, dtype=torch.uint32, device=ix.device)
    if out_scores is None:
        out_scores = torch.empty(B, k, dtype=torch.int32, device=ix.device)
    _check(lib().dessert_search(ix.handle, q_vectors.data_ptr(), ql.ctypes.data, B, _ptr(cand_ids),
                                None if co is None else co.ctypes.data, k, workspace.data_ptr(), workspace.numel(),
                                out_ids.data_ptr(), out_scores.data_ptr()))
    return out_ids, out_scores


def search_noalloc(ix: Index, q_vectors: torch.Tensor, q_length: int, k: int, cand_ids: Optional[torch.Tensor] = None,
                   out_ids: Optional[torch.Tensor] = None, out_scores: Optional[torch.Tensor] = None):
    """dessert_search_noalloc: query sets of q_length vectors each, candidate lists [B, cand_length] (or None: every
    document); the library's built-in scratch array is the workspace.  Outputs are allocated here only if not given."""
    q_vectors = _check_vectors(ix, q_vectors)
    if q_length <= 0 or q_vectors.shape[0] % q_length:
        raise ValueError("the number of query vectors must be a multiple of q_length")
    B = q_vectors.shape[0] // q_length
    cand_len = 0
    if cand_ids is not None:
        if cand_ids.dim() != 2 or cand_ids.shape[0] != B or cand_ids.dtype not in (torch.int32, torch.uint32):
            raise ValueError("cand_ids must be a device tensor [B, cand_length] of int32 / uint32")
        cand_ids = cand_ids.contiguous()
        cand_len = cand_ids.shape[1]
    if out_ids is None:
        out_ids = torch.empty(B, k, dtype=torch.uint32, device=ix.device)
    if out_scores is None:
        out_scores = torch.empty(B, k, dtype=torch.int32, device=ix.device)
    _check(lib().dessert_search_noalloc(ix.handle, q_vectors.data_ptr(), q_length, B, _ptr(cand_ids), cand_len, k,
                                        out_ids.data_ptr(), out_scores.data_ptr()))
    return out_ids, out_scores


def noalloc_scratch_bytes() -> int:
    return int(lib().dessert_noalloc_scratch_bytes())


def last_score_kernel(ix: Index) -> str:
    return lib().dessert_last_score_kernel(ix.handle).decode()


def set_debug(ix: Index, enable: bool = True) -> None:
    _check(lib().dessert_set_debug(ix.handle, int(bool(enable))))


def scores(ix: Index, q_vectors: torch.Tensor, q_lengths, cand_ids: Optional[torch.Tensor] = None,
           cand_offsets=None, workspace: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None):
    """dessert_scores: raw int32 scores, [total candidates] or [B, n_docs]."""
    q_vectors, ql, B, cand_ids, co, total = _batch(ix, q_vectors, q_lengths, cand_ids, cand_offsets)
    if workspace is None:
        workspace = torch.empty(workspace_bytes(ix, B, q_vectors.shape[0], total, 0), dtype=torch.uint8,
                                device=ix.device)
    if out is None:
        out = torch.empty(total, dtype=torch.int32, device=ix.device)
    _check(lib().dessert_scores(ix.handle, q_vectors.data_ptr(), ql.ctypes.data, B, _ptr(cand_ids),
                                None if co is None else co.ctypes.data, workspace.data_ptr(), workspace.numel(),
                                out.data_ptr()))
    return out if co is not None else out.view(B, ix.n_docs)


def filter_kmeans(ix: Index, sample: torch.Tensor, init_centroids: torch.Tensor, iterations: int) -> torch.Tensor:
    """dessert_filter_kmeans: Lloyd iterations from init_centroids on the sample; returns the new centroids [K, d] int8."""
    sample = _check_vectors(ix, sample)
    if not init_centroids.is_cuda or init_centroids.dtype != torch.int8 or init_centroids.dim() != 2 \
            or init_centroids.shape[1] != ix.cfg.d:
        raise ValueError("init_centroids must be a device int8 tensor [K, d]")
    cent = init_centroids.contiguous().clone()
    K, n = cent.shape[0], sample.shape[0]
    nbytes = int(lib().dessert_filter_kmeans_workspace_bytes(ix.handle, n, K))
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=ix.device)
    _check(lib().dessert_filter_kmeans(ix.handle, sample.data_ptr(), n, cent.data_ptr(), K, iterations,
                                       ws.data_ptr(), ws.numel()))
    return cent


def filter_build(ix: Index, centroids: torch.Tensor, vectors: torch.Tensor):
    """dessert_filter_build.  Returns (assign [V] int32, bucket_offsets [K+1] int32, bucket_docs [V] int32);
    only bucket_docs[: bucket_offsets[-1]] is meaningful."""
    vectors = _check_vectors(ix, vectors)
    if not centroids.is_cuda or centroids.dtype != torch.int8 or centroids.dim() != 2 or centroids.shape[1] != ix.cfg.d:
        raise ValueError("centroids must be a device int8 tensor [K, d]")
    centroids = centroids.contiguous()
    K, V = centroids.shape[0], vectors.shape[0]
    assign = torch.empty(V, dtype=torch.int32, device=ix.device)
    bucket_offsets = torch.empty(K + 1, dtype=torch.int32, device=ix.device)
    bucket_docs = torch.empty(max(V, 1), dtype=torch.int32, device=ix.device)
    _check(lib().dessert_filter_build(ix.handle, centroids.data_ptr(), K, vectors.data_ptr(), assign.data_ptr(),
                                      bucket_offsets.data_ptr(), bucket_docs.data_ptr()))
    ix._keep = [bucket_offsets, bucket_docs]
    return assign, bucket_offsets, bucket_docs


def filter_query(ix: Index, q_vectors: torch.Tensor, q_lengths, filter_probe: int, filter_k: int,
                 workspace: Optional[torch.Tensor] = None):
    """dessert_filter_query.  Returns (ids [B, filter_k] uint32 with 0xFFFFFFFF padding, counts [B, filter_k] int32)."""
    q_vectors = _check_vectors(ix, q_vectors)
    ql = _host_u32(q_lengths)
    B = ql.shape[0]
    if int(ql.sum()) != q_vectors.shape[0]:
        raise ValueError("sum(q_lengths) != number of query vectors")
    if workspace is None:
        nbytes = int(lib().dessert_filter_workspace_bytes(ix.handle, B, q_vectors.shape[0], int(ql.max()), filter_probe))
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=ix.device)
    ids = torch.empty(B, filter_k, dtype=torch.uint32, device=ix.device)
    counts = torch.empty(B, filter_k, dtype=torch.int32, device=ix.device)
    _check(lib().dessert_filter_query(ix.handle, q_vectors.data_ptr(), ql.ctypes.data, B, filter_probe, filter_k,
                                      workspace.data_ptr(), workspace.numel(), ids.data_ptr(), counts.data_ptr()))
    return ids, counts


def filter_search(ix: Index, q_vectors: torch.Tensor, q_lengths, filter_probe: int, filter_k: int, k: int,
                  workspace: Optional[torch.Tensor] = None, out_ids: Optional[torch.Tensor] = None,
                  out_scores: Optional[torch.Tensor] = None):
    """dessert_filter_search: filter, then search among the filter's candidates.  Returns (ids [B, k] uint32, scores [B, k] int32)."""
    q_vectors = _check_vectors(ix, q_vectors)
    ql = _host_u32(q_lengths)
    B = ql.shape[0]
    if int(ql.sum()) != q_vectors.shape[0]:
        raise ValueError("sum(q_lengths) != number of query vectors")
    if workspace is None:
        nbytes = int(lib().dessert_filter_search_workspace_bytes(ix.handle, B, q_vectors.shape[0], int(ql.max()) if B else 0,
                                                                 filter_probe, filter_k, k))
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=ix.device)
    if out_ids is None:
        out_ids = torch.empty(B, k, dtype=torch.uint32, device=ix.device)
    if out_scores is None:
        out_scores = torch.empty(B, k, dtype=torch.int32, device=ix.device)
    _check(lib().dessert_filter_search(ix.handle, q_vectors.data_ptr(), ql.ctypes.data, B, filter_probe, filter_k, k,
                                       workspace.data_ptr(), workspace.numel(), out_ids.data_ptr(), out_scores.data_ptr()))
    return out_ids, out_scores


def enable_timing(ix: Index, enable=True) -> None:
    """dessert_enable_timing: False/0 off, True/1 every call, n > 1 every n-th call."""
    _check(lib().dessert_enable_timing(ix.handle, int(enable)))


def get_timing(ix: Index, calls_back: int = 0):
    ms = (C.c_float * 4)()
    _check(lib().dessert_get_timing(ix.handle, calls_back, ms))
    return {"hash_ms": ms[0], "score_ms": ms[1], "topk_ms": ms[2], "total_ms": ms[3]}


def probe_read_bandwidth(buf: torch.Tensor, reps: int = 10) -> float:
    """dessert_probe_read_bandwidth: GB/s of a plain streaming read over `buf` (measurement aid)."""
    ms = C.c_float()
    nbytes = buf.numel() * buf.element_size()
    stream = torch.cuda.current_stream(buf.device).cuda_stream
    _check(lib().dessert_probe_read_bandwidth(buf.data_ptr(), nbytes, buf.device.index or 0, stream, reps, C.byref(ms)))
    return nbytes / (ms.value * 1e-3) / 1e9


def probe_mix_bandwidth(src: torch.Tensor, dst: torch.Tensor, reps: int = 10) -> float:
    """dessert_probe_mix_bandwidth: GB/s (read + written) of a kernel that reads 4 bytes of `src` for every byte it
    writes to `dst` and computes nothing (measurement aid: the ceiling for the index build's traffic)."""
    out_bytes = dst.numel() * dst.element_size()
    if src.numel() * src.element_size() < 4 * out_bytes:
        raise ValueError("src must hold four times the bytes of dst")
    ms = C.c_float()
    stream = torch.cuda.current_stream(dst.device).cuda_stream
    _check(lib().dessert_probe_mix_bandwidth(src.data_ptr(), dst.data_ptr(), out_bytes, dst.device.index or 0, stream, reps,
                                             C.byref(ms)))
    return 5 * out_bytes / (ms.value * 1e-3) / 1e9
