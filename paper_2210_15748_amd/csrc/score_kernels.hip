// Scoring kernels for gfx950: Alg. 2's loop over documents, query vectors and
// tables with sigma = max and A = sum,
//     score(Q,S) = sum_{q in Q} max_{x in S} #{ t : code_t(q) == code_t(x) }.
// Scores are raw integer counts (no division by L, no remap of Eq. 1).
#include "kernels.hpp"

#include <cstdio>

namespace dessert {

typedef int v4i __attribute__((ext_vector_type(4)));

// Where query set b's documents and outputs live.
struct Span {
    uint64_t base;   // first output slot (and first candidate entry)
    uint64_t count;  // documents scored by this query set
};

__device__ inline Span query_span(const ScoreArgs& a, uint32_t b) {
    Span s;
    if (a.cand_ids) {
        s.base = cand_begin(a, b);
        s.count = cand_begin(a, b + 1) - s.base;
    } else {
        s.base = (uint64_t)b * a.n_docs;
        s.count = a.n_docs;
    }
    return s;
}

// ---------------------------------------------------------------------------
// Code-compare kernel (plain form; any L that makes a code row a multiple of 4 bytes).
// CW = bytes per table code: 1 (C <= 8) or 2 (C <= 16).
// One wave per scored document; lanes stride over the document's vectors.  For
// each query vector the lane counts equal codes one dword at a time: z = q ^ x has a
// zero byte (halfword) exactly where the codes agree, and
//     nz = (((z & 0x7f7f7f7f) + 0x7f7f7f7f) | z) & 0x80808080
// has the top bit of a byte set exactly where z's byte is non-zero (0x7fff7fff / 0x80008000
// for halfwords).
template <int CW>
__global__ __launch_bounds__(256) void score_bytecmp_kernel(ScoreArgs a) {
    extern __shared__ uint32_t sq[];  // query set's codes, [mq][row dwords], then the phi table [L+1]
    constexpr uint32_t LOW = CW == 1 ? 0x7f7f7f7fu : 0x7fff7fffu;
    constexpr uint32_t TOP = CW == 1 ? 0x80808080u : 0x80008000u;
    constexpr int PER = 4 / CW;  // codes per dword
    const uint32_t b = blockIdx.y;
    const Span sp = query_span(a, b);
    const uint32_t q_lo = q_begin(a, b), mq = q_begin(a, b + 1) - q_lo;
    const uint32_t row = a.L * CW;  // bytes per code row
    const uint32_t LW = row / 4;
    const uint32_t* qsrc = (const uint32_t*)(a.qcodes + (size_t)q_lo * row);
    for (uint32_t i = threadIdx.x; i < mq * LW; i += blockDim.x) sq[i] = qsrc[i];
    uint32_t* tab = sq + (size_t)a.max_q_len * LW;
    if (a.remap)
        for (uint32_t i = threadIdx.x; i <= a.L; i += blockDim.x) tab[i] = a.remap[i];
    __syncthreads();

    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (uint64_t pos = (uint64_t)blockIdx.x * 4 + wave; pos < sp.count; pos += (uint64_t)gridDim.x * 4) {
        const uint64_t id = a.cand_ids ? a.cand_ids[sp.base + pos] : pos;
        if (a.cand_ids && id == 0xFFFFFFFFull) {  // empty candidate slot
            if (lane == 0) a.scores[sp.base + pos] = -1;
            continue;
        }
        const uint64_t lo = a.offsets[id], hi = a.offsets[id + 1];
        const uint64_t m = hi - lo;
        int32_t score = 0;
        for (uint32_t q = 0; q < mq; ++q) {
            int32_t best = 0;
            uint64_t sum = 0;  // sigma = mean: sum of phi over this lane's vectors
            for (uint64_t j = lo + lane; j < hi; j += 64) {
                const uint32_t* x = (const uint32_t*)(a.codes + j * row);
                int32_t cnt = 0;
                for (uint32_t w = 0; w < LW; ++w) {
                    uint32_t z = x[w] ^ sq[q * LW + w];
                    uint32_t nz = (((z & LOW) + LOW) | z) & TOP;
                    cnt += PER - __builtin_popcount(nz);
                }
                best = cnt > best ? cnt : best;
                if (a.sigma_mean) sum += tab[cnt];
            }
            uint32_t sg;
            if (a.sigma_mean) {
                for (int off = 32; off >= 1; off >>= 1) sum += (uint64_t)__shfl_xor((long long)sum, off, 64);
                sg = m ? (uint32_t)((sum + m / 2) / m) : 0u;
            } else {
                for (int off = 32; off >= 1; off >>= 1) {
                    int32_t o = __shfl_xor(best, off, 64);
                    best = o > best ? o : best;
                }
                sg = a.remap ? tab[best] : (uint32_t)best;
            }
            if (a.q_weights) sg = (uint32_t)(((uint64_t)a.q_weights[q_lo + q] * sg + 32768) >> 16);
            score += (int32_t)sg;
        }
        if (lane == 0) a.scores[sp.base + pos] = score;
    }
}

hipError_t launch_score_bytecmp(const ScoreArgs& a, hipStream_t stream, char* desc, size_t desc_len) {
    if (desc && desc_len) desc[0] = 0;
    if (a.n_queries == 0 || a.max_scored == 0) return hipSuccess;
    if ((a.code_bytes != 1 && a.code_bytes != 2) || (a.L * a.code_bytes) % 4) return hipErrorInvalidValue;
    if (a.sigma_mean && !a.remap) return hipErrorInvalidValue;
    size_t lds = (size_t)a.max_q_len * a.L * a.code_bytes + ((size_t)a.L + 1) * 4;
    if (lds > 65536 + 1024) return hipErrorInvalidValue;
    if (lds > 48 * 1024) {
        static hipError_t a1 = hipFuncSetAttribute((const void*)score_bytecmp_kernel<1>,
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, 65536 + 1024);
        static hipError_t a2 = hipFuncSetAttribute((const void*)score_bytecmp_kernel<2>,
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, 65536 + 1024);
        if (a1 != hipSuccess) return a1;
        if (a2 != hipSuccess) return a2;
    }
    uint64_t bx = (a.max_scored + 3) / 4;
    if (bx > 4096) bx = 4096;
    if (desc) snprintf(desc, desc_len, "score_bytecmp_kernel<%u>", a.code_bytes);
    if (a.code_bytes == 1)
        hipLaunchKernelGGL(score_bytecmp_kernel<1>, dim3((unsigned)bx, a.n_queries), dim3(256), lds, stream, a);
    else
        hipLaunchKernelGGL(score_bytecmp_kernel<2>, dim3((unsigned)bx, a.n_queries), dim3(256), lds, stream, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Mask-table kernel: bit-parallel over the query vectors.
//
// For a chunk of up to 32 query vectors the workgroup builds, in LDS,
//     M[t][h] = { q : code_t(q) == h }   as a 32-bit mask,
// so one LDS read M[t][code_t(x)] answers "which q collide with x in table t"
// for all 32 q at once.  A lane owns one document vector x at a time: it reads
// the L masks of x, adds them with a carry-save adder tree into a bit-sliced
// counter (plane p holds bit p of cnt(q,x) for the 32 q), and folds that into
// a bit-sliced running maximum.  Eight lanes share a document; at its end
// their maxima are merged with DPP lane exchanges and the score is
//     sum_q max_x cnt(q,x) = sum_p 2^p * popcount(plane_p).
// Everything is integer and exact.  Query sets longer than 32 vectors are
// processed in chunks of 32 whose partial sums add (the score is a sum over q).

// three-input boolean functions through v_bitop3_b32; the immediate is the
// function's truth table evaluated on a=0xF0, b=0xCC, c=0xAA
#define DESSERT_BITOP3(a, b, c, tt) __builtin_amdgcn_bitop3_b32((a), (b), (c), (tt))
__device__ inline uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) { return DESSERT_BITOP3(a, b, c, 0x96); }
__device__ inline uint32_t maj3(uint32_t a, uint32_t b, uint32_t c) { return DESSERT_BITOP3(a, b, c, 0xE8); }
// borrow out of a - b with borrow-in c: maj(~a, b, c)
__device__ inline uint32_t borrow3(uint32_t a, uint32_t b, uint32_t c) { return DESSERT_BITOP3(a, b, c, 0x8E); }
// sel ? x : y, bitwise
__device__ inline uint32_t select3(uint32_t sel, uint32_t x, uint32_t y) { return DESSERT_BITOP3(sel, x, y, 0xCA); }

// Sum N one-bit-per-position inputs into bit planes: planes[p] = bit p of the
// per-position count.  Inputs of one weight are consumed three at a time by
// full adders (sum stays at the weight and re-enters the queue, carry moves to
// the next weight); an even count ends with one half adder.
template <int N>
__device__ inline void csa_planes(const uint32_t* in, uint32_t* planes) {
    if constexpr (N == 1) {
        planes[0] = in[0];
    } else {
        constexpr int F = (N - 1) / 2;  // full adders at this weight
        uint32_t w[N + F];
        uint32_t next[N / 2];
#pragma unroll
        for (int i = 0; i < N; ++i) w[i] = in[i];
#pragma unroll
        for (int f = 0; f < F; ++f) {
            uint32_t x = w[3 * f], y = w[3 * f + 1], z = w[3 * f + 2];
            w[N + f] = xor3(x, y, z);
            next[f] = maj3(x, y, z);
        }
        if constexpr (N % 2 == 0) {
            uint32_t x = w[N + F - 2], y = w[N + F - 1];
            planes[0] = x ^ y;
            next[N / 2 - 1] = x & y;
        } else {
            planes[0] = w[N + F - 1];
        }
        csa_planes<N / 2>(next, planes + 1);
    }
}

template <int P>
__device__ inline void planes_max(uint32_t* mx, const uint32_t* c) {
    // lt = (mx < c) per bit position, from the borrow chain of mx - c
    uint32_t lt = 0;
#pragma unroll
    for (int p = 0; p < P; ++p) lt = borrow3(mx[p], c[p], lt);
#pragma unroll
    for (int p = 0; p < P; ++p) mx[p] = select3(lt, c[p], mx[p]);
}

// acc (WA planes) += b (WB planes) per bit position: a ripple of full adders over b's planes, then of half adders
template <int WA, int WB>
__device__ inline void planes_add(uint32_t* acc, const uint32_t* b) {
    static_assert(WB <= WA, "the addend is not wider than the accumulator");
    uint32_t carry = 0;
#pragma unroll
    for (int p = 0; p < WB; ++p) {
        const uint32_t x = acc[p];
        acc[p] = xor3(x, b[p], carry);
        carry = maj3(x, b[p], carry);
    }
#pragma unroll
    for (int p = WB; p < WA; ++p) {
        const uint32_t x = acc[p];
        acc[p] = x ^ carry;
        carry = x & carry;
    }
}

template <int CTRL>
__device__ inline uint32_t dpp_mov(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}

// byte K of dw shifted left by `sh` (the LDS byte offset of a table entry of 1 << sh bytes), in one
// SDWA shift; sh lives in a VGPR because SDWA takes no literal operand
template <int K>
__device__ inline uint32_t byte_shl(uint32_t dw, uint32_t sh) {
    uint32_t r;
    if constexpr (K == 0)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0"
            : "=v"(r) : "v"(sh), "v"(dw));
    else if constexpr (K == 1)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1"
            : "=v"(r) : "v"(sh), "v"(dw));
    else if constexpr (K == 2)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2"
            : "=v"(r) : "v"(sh), "v"(dw));
    else
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3"
            : "=v"(r) : "v"(sh), "v"(dw));
    return r;
}

// halfword K of dw shifted left by sh (16-bit codes)
template <int K>
__device__ inline uint32_t half_shl(uint32_t dw, uint32_t sh) {
    uint32_t r;
    if constexpr (K == 0)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0"
            : "=v"(r) : "v"(sh), "v"(dw));
    else
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1"
            : "=v"(r) : "v"(sh), "v"(dw));
    return r;
}

constexpr int ilog2_ceil(int x) { return x <= 1 ? 0 : 1 + ilog2_ceil((x + 1) / 2); }

constexpr uint32_t LUT_DOCS = 256;  // documents per workgroup (upper bound)
// Threads per workgroup: a mask table of 32 KB or more limits a CU to a few workgroups, so eight waves share
// one table instead of four: from 32 KB where the register budget allows it (few tables), always from 64 KB.
// The rotated table order (see below): one-byte codes, one query set per workgroup, 64 or 32 tables.
// With 32 tables only from 128 entries per table on: the rows of the rotated order are twice the size of the plain table,
// and the small tables (64 entries) measure faster plain.
constexpr bool masklut_rotated(int L, int CB, int CW, int W) { return (L == 64 || (L == 32 && CB >= 7)) && CW == 1 && W == 1; }
// Bytes of LDS the table takes: rows of the rotated order are 256 bytes (64 slots) also with 32 tables.
constexpr int masklut_table_bytes(int L, int CB, int CW, int W) { return masklut_rotated(L, CB, CW, W) ? (64 << CB) * 4 : (L << CB) * 4 * W; }
constexpr int masklut_threads(int L, int CB, int CW, int W) {
    return (masklut_table_bytes(L, CB, CW, W) >= 32 * 1024 &&
            (L <= 16 || L >= 128 || masklut_table_bytes(L, CB, CW, W) >= 64 * 1024)) ? 512 : 256;
}
// Waves per SIMD the register allocation must allow: the rotated form (L = 64) keeps 24 more per-lane
// constants and would otherwise drop from 4 to 3.
constexpr int masklut_min_waves(int L, int CB, int CW, int W, int REMAP) {
    if (L == 64 && CW == 1 && W == 1 && REMAP < 3) return 4;
    return 1;
}
constexpr uint32_t LUT_BINS = 64;   // length classes for the in-block ordering

// Per-workgroup bookkeeping, in static LDS beside the mask table.
struct LutBlockMeta {
    uint64_t lo[LUT_DOCS];      // first code row of each document of the block
    uint32_t m[LUT_DOCS];       // its length
    uint32_t slot[LUT_DOCS];    // its slot within the query set's candidate list (= output position)
    uint16_t order[LUT_DOCS];   // documents ordered longest class first
    uint32_t bin[LUT_BINS];     // counting sort by length class
    uint32_t next;              // next unclaimed position in `order`
};

// G = lanes per document: a wave works on 64/G documents at a time, each lane looping over
// every G-th vector of its document.  G = 8, except the paired form with L <= 32 (G = 4): there the work is
// vector-ALU arithmetic, and merging a document's lanes costs about as much as one round of the loop, so with
// documents of some 70 vectors fewer lanes per document (two merge steps, less rounding up to whole rounds)
// measured 4-6 % faster; with 64-byte rows (L = 64) it made no difference.  Documents of a block are ordered by length class
// ceil(m/G) (counting sort in LDS) and waves claim runs of 64/G consecutive documents from that
// order, so the documents sharing a wave need the same number of rounds and few lanes idle.
//
// W = query sets per workgroup.  W = 2 (only when every document is scored for every query set)
// stores the masks of two query sets side by side, M[t][h] = {mask of set 2y, mask of set 2y+1},
// so one 8-byte LDS read serves 64 query vectors: a random 8-byte read costs about 6.8 cycles
// per wave against 5.9 for a 4-byte one, and the code loads and address shifts are shared.
// REMAP: 1 = apply the fixed-point table a.remap (Eq. 1, or another phi) to each per-query-vector maximum;
// 2 = and weight the query vectors by a.q_weights (Sec. 4.2); 0 = raw counts.
// 3 / 4 = sigma is the MEAN over the document's vectors of phi(count / L) with phi the identity (Sec. 4.1, the lemma
// on sigma = (1/m) sum phi(x_i)), without / with weights: with L a power of two the Q16 table is 65536/L * count exactly,
// so what is needed per query vector is S = sum_x cnt(q,x).  The count planes of a round (zeroed in lanes that hold no
// row of the document) are added into a bit-sliced accumulator of P+4 planes, which every 16 rounds is added into one
// of P+15 planes; the lanes of a document add theirs over DPP, each lane un-slices its share of the query vectors and
// forms (65536/L * S + floor(m/2)) / m.  Needs documents shorter than 65536 vectors (32-bit numerators).
// CW = bytes per table code (1: C <= 8, 2: wider codes); CB = bits of a table index (2^CB entries per table).
// gz = chunk groups: with gz > 1 the 32-vector chunks of a query set are dealt round-robin to gz
// workgroups, which add their partial sums into the (pre-zeroed) scores with integer atomics.
// (SPLIT = false: gz is 1.)
//
// Rotated table order (L = 64, one-byte codes, one query set per workgroup).  LDS serves the 32 lanes of a
// half-wave in one pass when their dwords lie in 32 different banks (bank = dword address mod 32).  With
// M[t][h] the bank is the low bits of the code, i.e. random: a read takes about 2.4 passes, and with 64
// reads per document vector this form is bound by LDS.  Here the table is stored code-major, row h =
// the 64 masks {M[t][h]} at byte h * 256, and in any one read instruction the 32 lanes of a half-wave
// ask for 32 different tables whose positions differ mod 32, so whatever their codes are they address
// different banks.  A lane's read of register k (a dword of its code row), byte b, is for table
//     t = 4 * (k ^ r0 ^ 4*a) + ((b + rb) & 3):
//   a  (lane bits 2-3)  the lane loads the four 16-byte quarters of its code row in a permuted order;
//   r0 (lane bit 4)     neighbouring registers are exchanged (one select per register);
//   rb (lane bits 0-1)  the byte picked from the register is rotated - free, the byte index sits in
//                       the per-lane selector of the v_perm that forms the address.
// Table t sits at slot rot_slot(t) of a row: bit 1 of k, the one bit of t that the lanes of a read share,
// moved to the top.  The address (h << 8) | (4 * slot) is one v_perm: byte 1 from the code register,
// byte 0 from a per-lane constant.  (Measured on the fp16 stress preset: scoring 198 -> 102 ms.  The same
// order for paired L = 32 tables, 8-byte slots, was 7 % slower than M[t][h]: that form is bound by the
// vector ALU, not by LDS.)
// With 32 tables (one set per workgroup, 128 or 256 entries per table) the order is used too: candidate scoring with
// M[t][h] had LDS 95 % busy, 60 % of it conflicts, next to the memory reads it is bound by; rotated it is 3 % faster at
// C = 7 and 8 % at C = 8 (vector ALU 71 % -> 85 % busy: the selects and the permuted loads).
__device__ inline uint32_t rot_slot(uint32_t k, uint32_t b) {  // k = (k3 k2 k1 k0): slot (k1 k3 k2 k0 b1 b0)
    return ((k >> 1) & 1) * 32 + ((k >> 3) & 1) * 16 + ((k >> 2) & 1) * 8 + (k & 1) * 4 + b;
}
// L = 32: a row has room for the 32 masks twice, and a row has to start on a multiple of 256 bytes anyway for the
// one-v_perm address.  Slots 0..31 hold table t at slot t, slots 32..63 hold table t at slot 32 + (t ^ 8).  The eight
// registers of a code row are permuted by two lane bits (the two 16-byte halves by the load order, neighbouring
// registers by one select), the bytes by two more, and the fifth bit of the lane picks the copy: in any read the 16
// lanes that use the first copy ask for 16 different tables, the 16 lanes of the second copy for the same 16 tables,
// whose slots there have bit 3 flipped, so the 32 lanes still address 32 different banks.
template <int L>
__device__ inline uint32_t rot_slot_of(uint32_t k, uint32_t b) { return L == 64 ? rot_slot(k, b) : 4 * k + b; }

template <int L, int CB, int CW, int REMAP, int W, bool SPLIT>
__global__ __launch_bounds__(masklut_threads(L, CB, CW, W), masklut_min_waves(L, CB, CW, W, REMAP)) void score_masklut_kernel(ScoreArgs a, uint32_t docs_per_block, uint32_t gy_linear,
                                                            uint32_t gz_arg) {
    constexpr bool ROT = masklut_rotated(L, CB, CW, W);
    const uint32_t gz = SPLIT ? gz_arg : 1u;
    constexpr int T = masklut_threads(L, CB, CW, W);
    constexpr int LW = L * CW / 4;  // dwords per code row
    constexpr int STRIDE = 1 << CB;
    constexpr int P = ilog2_ceil(L + 1);  // planes needed for counts 0..L
    constexpr int G = (W == 2 && L <= 32) ? 4 : 8;
    constexpr int DOCS_PER_WAVE = 64 / G;
    constexpr bool MEAN = REMAP >= 3;
    constexpr bool WEIGHTED = REMAP == 2 || REMAP == 4;
    constexpr int P1 = P + 4;    // planes of the 16-round accumulator: 16 * L < 2^(P+4)
    constexpr int P2 = P + 15;   // planes of the document's accumulator: S <= L * m < 2^(P-1) * 2^16
    // static LDS: the table sits at a link-time constant address, so t*STRIDE*4*W folds into the
    // immediate offset of each ds_read and the only per-read address arithmetic is one shift
    constexpr int LUT_WORDS = masklut_table_bytes(L, CB, CW, W) / 4;
    __shared__ __attribute__((aligned(256))) uint32_t lut[LUT_WORDS];  // [t][h][w]; ROT: [h][pos(t)]
    __shared__ LutBlockMeta meta;

    // Which (document block, query-set group) this workgroup takes.  When every set scores every
    // document (gy_linear != 0) the grid is linear and decoded so that the groups of one document
    // block run back to back on ONE XCD (workgroup ids go round-robin over the 8 XCDs): the
    // block's codes then come from HBM once and from that XCD's L2 for the other groups.
    uint32_t bx_idx, by_idx;
    if (gy_linear) {
        const uint32_t xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
        by_idx = j % gy_linear;
        bx_idx = (j / gy_linear) * 8 + xcd;
    } else {
        bx_idx = blockIdx.x;
        by_idx = blockIdx.y;
    }
    const uint32_t cz = SPLIT ? by_idx % gz : 0u;  // chunk group
    if constexpr (SPLIT) by_idx /= gz;
    const uint32_t b0 = by_idx * W;     // first query set of this workgroup
    const Span sp = query_span(a, b0);  // W > 1: every set scores the same documents
    const uint64_t first = (uint64_t)bx_idx * docs_per_block;
    if (first >= sp.count) return;
    const uint32_t ndocs = (uint32_t)((first + docs_per_block < sp.count) ? docs_per_block : sp.count - first);
    uint32_t q_lo[W], q_len[W], max_len = 0;
#pragma unroll
    for (int w = 0; w < W; ++w) {
        const bool have = b0 + w < a.n_queries;
        q_lo[w] = have ? q_begin(a, b0 + w) : 0;
        q_len[w] = have ? q_begin(a, b0 + w + 1) - q_lo[w] : 0;
        max_len = q_len[w] > max_len ? q_len[w] : max_len;
    }
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t sub = lane & (G - 1);  // lane within the document's group
    const uint32_t grp = lane / G;        // group within the wave

    // ---- prologue: where each document lives, the length-class ordering, and the first chunk's mask
    // table.  Global loads are issued first and used late, so the dependent chain candidate id ->
    // offsets runs while the table is zeroed and the query codes arrive.
    const uint32_t c_first = cz * 32;  // first chunk of 32 query vectors taken by this workgroup
    auto chunk_len = [&](int w, uint32_t c0) { return c0 >= q_len[w] ? 0u : (q_len[w] - c0 < 32 ? q_len[w] - c0 : 32u); };
    auto query_code = [&](int w, uint32_t c0, uint32_t i) {  // entry i = (q, t) of the chunk: the code of q in table t
        const size_t at = (size_t)(q_lo[w] + c0) * L + i;
        return CW == 1 ? (uint32_t)a.qcodes[at] : (uint32_t)((const uint16_t*)a.qcodes)[at];
    };
    auto table_or = [&](int w, uint32_t i, uint32_t h) {
        const uint32_t q = i / L, t = i % L;
        if constexpr (ROT) {
            atomicOr(&lut[h * 64 + rot_slot_of<L>(t >> 2, t & 3)], 1u << q);
            if constexpr (L == 32) atomicOr(&lut[h * 64 + 32 + (t ^ 8)], 1u << q);  // the second copy
        }
        else atomicOr(&lut[(t * STRIDE + h) * W + w], 1u << q);
    };
    auto zero_table = [&]() {
        for (uint32_t i = threadIdx.x; i < LUT_WORDS; i += T) lut[i] = 0;
    };
    const bool have_doc = threadIdx.x < ndocs;
    uint64_t my_id = 0;
    uint32_t my_slot = 0;
    if (have_doc) {
        const uint64_t pos = first + threadIdx.x;
        my_slot = (uint32_t)(a.order ? a.order[sp.base + pos] : pos);  // a.order: candidate mode only
        my_id = a.cand_ids ? a.cand_ids[sp.base + my_slot] : pos;
    }
    constexpr int QPT = (32 * L + T - 1) / T;  // table entries per thread and query set
    uint32_t qh[W][QPT];
#pragma unroll
    for (int w = 0; w < W; ++w) {
        const uint32_t n_ent = chunk_len(w, c_first) * L;
#pragma unroll
        for (int n = 0; n < QPT; ++n) {
            const uint32_t i = threadIdx.x + n * T;
            qh[w][n] = i < n_ent ? query_code(w, c_first, i) : 0u;
        }
    }
    zero_table();
    for (uint32_t i = threadIdx.x; i < LUT_BINS; i += T) meta.bin[i] = 0;
    if (threadIdx.x == 0) meta.next = 0;
    // an empty candidate slot (id 0xFFFFFFFF) is kept as a zero-length document whose stored
    // start is all ones; it is written as score -1 below
    const bool empty_slot = a.cand_ids && my_id == 0xFFFFFFFFull;
    uint64_t my_lo = ~0ull, my_hi = ~0ull;
    if (have_doc && !empty_slot) {
        my_lo = a.offsets[my_id];
        my_hi = a.offsets[my_id + 1];
    }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < W; ++w) {
        const uint32_t n_ent = chunk_len(w, c_first) * L;
#pragma unroll
        for (int n = 0; n < QPT; ++n) {
            const uint32_t i = threadIdx.x + n * T;
            if (i < n_ent) table_or(w, i, qh[w][n]);
        }
    }
    uint32_t my_class = 0;
    if (have_doc) {
        const uint32_t m = (uint32_t)(my_hi - my_lo);  // 0 for an empty slot
        meta.lo[threadIdx.x] = my_lo;
        meta.m[threadIdx.x] = m;
        meta.slot[threadIdx.x] = a.order ? my_slot : (uint32_t)(first + threadIdx.x);
        uint32_t rounds = (m + G - 1) / G;
        my_class = rounds < LUT_BINS ? LUT_BINS - 1 - rounds : 0;  // class 0 = longest
        atomicAdd(&meta.bin[my_class], 1u);
    }
    __syncthreads();
    if (threadIdx.x < 64) {  // exclusive scan of the 64 class counts by one wave
        uint32_t c = meta.bin[lane], incl = c;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            uint32_t o = __shfl_up(incl, off, 64);
            if ((int)lane >= off) incl += o;
        }
        meta.bin[lane] = incl - c;
    }
    __syncthreads();
    if (have_doc) meta.order[atomicAdd(&meta.bin[my_class], 1u)] = (uint16_t)threadIdx.x;

    const uint32_t entry_shift = W == 1 ? 2 : 3;  // log2 of the bytes per table entry
    // ROT: lane-dependent table order (see above)
    uint32_t rot_sel[4], rot_posc[ROT ? LW : 1], rot_quarter[ROT ? LW / 4 : 1], rot_swap = 0;
    if constexpr (ROT) {
        // lane bits 0-1: byte rotation; then L = 64: bits 2-3 quarter order, bit 4 neighbour exchange;
        // L = 32: bit 2 neighbour exchange, bit 3 which copy of the masks, bit 4 order of the two halves
        const uint32_t rb = lane & 3;
        const uint32_t aq = L == 64 ? (lane >> 2) & 3 : (lane >> 4) & 1;
        const uint32_t r0 = L == 64 ? (lane >> 4) & 1 : (lane >> 2) & 1;
        const uint32_t copy = L == 64 ? 0u : (lane >> 3) & 1;
        rot_swap = r0 ? ~0u : 0u;
#pragma unroll
        for (int b = 0; b < 4; ++b) rot_sel[b] = 0x0c0c0000u | ((4 + ((b + rb) & 3)) << 8) | b;
#pragma unroll
        for (int q = 0; q < LW / 4; ++q) rot_quarter[q] = 16 * (q ^ aq);  // byte offset of the piece loaded into registers 4q..4q+3
#pragma unroll
        for (int k = 0; k < LW; ++k) {
            rot_posc[k] = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b)
            {
                const uint32_t slot = rot_slot_of<L>(k ^ r0 ^ (aq << 2), (b + rb) & 3);
                rot_posc[k] |= ((copy ? 32 + (slot ^ 8) : slot) * 4) << (8 * b);
            }
        }
        // keep the per-lane constants in registers (otherwise they are rebuilt inside the loop)
#pragma unroll
        for (int b = 0; b < 4; ++b) asm volatile("" : "+v"(rot_sel[b]));
#pragma unroll
        for (int q = 0; q < LW / 4; ++q) asm volatile("" : "+v"(rot_quarter[q]));
#pragma unroll
        for (int k = 0; k < LW; ++k) asm volatile("" : "+v"(rot_posc[k]));
        asm volatile("" : "+v"(rot_swap));
    }
    for (uint32_t c0 = c_first; c0 < max_len; c0 += gz * 32) {  // chunks of 32 query vectors
        if (c0 != c_first) {  // the first chunk's table was built above
            __syncthreads();  // previous chunk's readers are done
            zero_table();
            if (threadIdx.x == 0) meta.next = 0;
            __syncthreads();
#pragma unroll
            for (int w = 0; w < W; ++w) {
                const uint32_t n_ent = chunk_len(w, c0) * L;
                for (uint32_t i = threadIdx.x; i < n_ent; i += T) table_or(w, i, query_code(w, c0, i));
            }
        }
        __syncthreads();  // table and `order` complete

        for (;;) {
            uint32_t claim = 0;
            if (lane == 0) claim = atomicAdd(&meta.next, (uint32_t)DOCS_PER_WAVE);
            claim = __builtin_amdgcn_readfirstlane(claim);
            if (claim >= ndocs) break;
            const uint32_t slot = claim + grp;
            const bool valid = slot < ndocs;
            const uint32_t doc = valid ? meta.order[slot] : 0;
            const uint32_t m = valid ? meta.m[doc] : 0;
            // groups with nothing to do read row 0 (the caller guarantees the index holds a vector)
            const uint64_t lo = m ? meta.lo[doc] : 0;
            const uint32_t last_j = m ? m - 1 : 0;

            uint32_t mx[W][MEAN ? 1 : P];          // running maximum (sigma = max)
            uint32_t sum1[W][MEAN ? P1 : 1];       // sums of the last few rounds, and of the document (sigma = mean)
            uint32_t sum2[W][MEAN ? P2 : 1];
            uint32_t rounds_in_sum1 = 0;
#pragma unroll
            for (int w = 0; w < W; ++w) {
#pragma unroll
                for (int p = 0; p < (MEAN ? 1 : P); ++p) mx[w][p] = 0;
#pragma unroll
                for (int p = 0; p < (MEAN ? P1 : 1); ++p) sum1[w][p] = 0;
#pragma unroll
                for (int p = 0; p < (MEAN ? P2 : 1); ++p) sum2[w][p] = 0;
            }

            // lanes past the end re-read the document's last vector (a repeated vector cannot
            // change the maximum); the next round's codes are requested before this round's
            // table reads so that HBM latency overlaps the bit-sliced arithmetic
            const uint8_t* doc_codes = a.codes + lo * (L * CW);
            auto load_codes = [&](int32_t j, uint32_t (&dst)[LW]) {  // j: row within the document, already clamped
                const uint8_t* row = doc_codes + (uint32_t)j * (uint32_t)(L * CW);
                if constexpr (ROT) {
#pragma unroll
                    for (int q = 0; q < LW / 4; ++q) {
                        const v4i v = *(const v4i*)(doc_codes + ((uint32_t)j * (uint32_t)(L * CW) + rot_quarter[q]));
                        dst[4 * q] = v.x; dst[4 * q + 1] = v.y; dst[4 * q + 2] = v.z; dst[4 * q + 3] = v.w;
                    }
                } else if constexpr (LW % 4 == 0) {
                    const v4i* src = (const v4i*)row;
#pragma unroll
                    for (int w = 0; w < LW; w += 4) {
                        v4i v = src[w / 4];
                        dst[w] = v.x; dst[w + 1] = v.y; dst[w + 2] = v.z; dst[w + 3] = v.w;
                    }
                } else {
                    static_assert(LW % 4 == 0 || LW == 2, "code rows of 8 or a multiple of 16 bytes");
                    uint2 v = *(const uint2*)row;
                    dst[0] = v.x; dst[1] = v.y;
                }
            };
            // one round: the table reads of this lane's vector, the carry-save count and the running maximum (or sum).
            // row = the lane's row of the document in this round before clamping: only rows 0 .. m-1 count towards a sum
            auto process = [&](const uint32_t (&dw)[LW], int32_t row) {
                const char* lut_bytes = reinterpret_cast<const char*>(lut);
                uint32_t off[L];  // byte offset of x's entry within each table
#pragma unroll
                for (int w = 0; w < LW; ++w) {
                    if constexpr (ROT) {
                        const uint32_t v = select3(rot_swap, dw[w ^ 1], dw[w]);
#pragma unroll
                        for (int b = 0; b < 4; ++b) off[4 * w + b] = __builtin_amdgcn_perm(v, rot_posc[w], rot_sel[b]);
                    } else if constexpr (CW == 1) {
                        off[4 * w + 0] = byte_shl<0>(dw[w], entry_shift);
                        off[4 * w + 1] = byte_shl<1>(dw[w], entry_shift);
                        off[4 * w + 2] = byte_shl<2>(dw[w], entry_shift);
                        off[4 * w + 3] = byte_shl<3>(dw[w], entry_shift);
                    } else {
                        off[2 * w + 0] = half_shl<0>(dw[w], entry_shift);
                        off[2 * w + 1] = half_shl<1>(dw[w], entry_shift);
                    }
                }
                uint32_t msk[W][L];
#pragma unroll
                for (int t = 0; t < L; ++t) {
                    if constexpr (ROT) {
                        msk[0][t] = *(const uint32_t*)(lut_bytes + off[t]);
                    } else if constexpr (W == 1) {
                        msk[0][t] = *(const uint32_t*)(lut_bytes + t * STRIDE * 4 + off[t]);
                    } else {
                        uint2 e = *(const uint2*)(lut_bytes + t * STRIDE * 8 + off[t]);
                        msk[0][t] = e.x;
                        msk[1][t] = e.y;
                    }
                }
#pragma unroll
                for (int w = 0; w < W; ++w) {
                    uint32_t cnt[P];
                    csa_planes<L>(msk[w], cnt);
                    if constexpr (!MEAN) {
                        planes_max<P>(mx[w], cnt);
                    } else {
                        const uint32_t keep = (row >= 0 && row < (int32_t)m) ? ~0u : 0u;
#pragma unroll
                        for (int p = 0; p < P; ++p) cnt[p] &= keep;
                        planes_add<P1, P>(sum1[w], cnt);
                    }
                }
                if constexpr (MEAN) {
                    if (++rounds_in_sum1 == 16) {   // the same for every lane of the wave
                        rounds_in_sum1 = 0;
#pragma unroll
                        for (int w = 0; w < W; ++w) {
                            planes_add<P2, P1>(sum2[w], sum1[w]);
#pragma unroll
                            for (int p = 0; p < P1; ++p) sum1[w][p] = 0;
                        }
                    }
                }
            };
            // a round's G rows start on a 128-byte line of the code array (rows before the document's
            // first clamp to it), so the rows of one round are whole lines and no line is requested
            // by two rounds.  Not in the paired form: it streams the code array in order and is bound by
            // arithmetic, so it starts at the document's first row and computes no clamped rows in front
            constexpr uint32_t ROWS_PER_LINE = W == 2 ? 1 : 128 / (L * CW) < 1 ? 1 : (128 / (L * CW) > G ? G : 128 / (L * CW));
            int32_t j = (int32_t)sub - (int32_t)((uint32_t)lo & (ROWS_PER_LINE - 1));  // this lane's row in the round at hand
            const int32_t j_end = (int32_t)m + (int32_t)sub;  // rounds run while j - sub < m
            auto clamped = [&](int32_t jj) { return jj < (int32_t)last_j ? jj : (int32_t)last_j; };
            // code buffers used in turn (the loop body is one round per buffer), so no register copies;
            // DEPTH rounds of codes are in flight while a round is processed
            constexpr int DEPTH = (W == 1 && LW <= 8) ? 2 : 1;
            if constexpr (DEPTH == 1) {
                uint32_t buf_a[LW], buf_b[LW];
                load_codes(clamped(j < 0 ? 0 : j), buf_a);
                for (;;) {
                    load_codes(clamped(j + G), buf_b);
                    process(buf_a, j);
                    j += G;
                    if (!__any(j < j_end)) break;
                    load_codes(clamped(j + G), buf_a);
                    process(buf_b, j);
                    j += G;
                    if (!__any(j < j_end)) break;
                }
            } else {
                uint32_t buf_a[LW], buf_b[LW], buf_c[LW];
                load_codes(clamped(j < 0 ? 0 : j), buf_a);
                load_codes(clamped(j + G), buf_b);
                for (;;) {
                    load_codes(clamped(j + 2 * G), buf_c);
                    process(buf_a, j);
                    j += G;
                    if (!__any(j < j_end)) break;
                    load_codes(clamped(j + 2 * G), buf_a);
                    process(buf_b, j);
                    j += G;
                    if (!__any(j < j_end)) break;
                    load_codes(clamped(j + 2 * G), buf_b);
                    process(buf_c, j);
                    j += G;
                    if (!__any(j < j_end)) break;
                }
            }
#pragma unroll
            for (int w = 0; w < W; ++w) {
                int32_t score = 0;
                if constexpr (!MEAN) {
                    if (m == 0) {  // empty document: the maximum over nothing is 0
#pragma unroll
                        for (int p = 0; p < P; ++p) mx[w][p] = 0;
                    }
                    // merge the G lanes of a document: (G = 8) mirror within the half row, then the two
                    // quad exchanges
                    uint32_t o[P];
                    if constexpr (G == 8) {
#pragma unroll
                        for (int p = 0; p < P; ++p) o[p] = dpp_mov<0x141>(mx[w][p]);  // row_half_mirror
                        planes_max<P>(mx[w], o);
                    }
#pragma unroll
                    for (int p = 0; p < P; ++p) o[p] = dpp_mov<0xB1>(mx[w][p]);   // quad_perm [1,0,3,2]
                    planes_max<P>(mx[w], o);
#pragma unroll
                    for (int p = 0; p < P; ++p) o[p] = dpp_mov<0x4E>(mx[w][p]);   // quad_perm [2,3,0,1]
                    planes_max<P>(mx[w], o);
                }
                if constexpr (REMAP == 0) {
#pragma unroll
                    for (int p = P - 1; p >= 0; --p) score = 2 * score + __builtin_popcount(mx[w][p]);
                } else if constexpr (!MEAN) {
                    // similarity remap (Eq. 1 as a table of L+1 fixed-point values): every lane of
                    // the group holds the merged maxima; lane `sub` un-slices query vectors sub,
                    // sub+8, sub+16, sub+24, looks their maxima up, and the eight partial sums are
                    // added (integers, so the order does not matter)
                    uint32_t part = 0;
#pragma unroll
                    for (int jq = 0; jq < 32 / G; ++jq) {
                        const uint32_t q = sub + G * jq;
                        uint32_t v = 0;
#pragma unroll
                        for (int p = P - 1; p >= 0; --p) v = 2 * v + ((mx[w][p] >> q) & 1u);
                        uint32_t term = a.remap[v];  // remap[0] = 0, and absent query vectors have maximum 0
                        if (WEIGHTED && c0 + q < q_len[w])
                            term = (uint32_t)(((uint64_t)a.q_weights[q_lo[w] + c0 + q] * term + 32768) >> 16);
                        part += term;
                    }
                    if constexpr (G == 8) part += dpp_mov<0x141>(part);  // row_half_mirror
                    part += dpp_mov<0xB1>(part);   // quad_perm [1,0,3,2]
                    part += dpp_mov<0x4E>(part);   // quad_perm [2,3,0,1]
                    score = (int32_t)part;
                } else {
                    // sigma = mean of count / L: the document's sums S(q) = sum_x cnt(q,x), first this lane's
                    // (what is left in the 16-round accumulator joins the document's), then the G lanes' by
                    // bit-sliced additions over the same lane exchanges as above
                    planes_add<P2, P1>(sum2[w], sum1[w]);
                    uint32_t o[P2];
                    if constexpr (G == 8) {
#pragma unroll
                        for (int p = 0; p < P2; ++p) o[p] = dpp_mov<0x141>(sum2[w][p]);
                        planes_add<P2, P2>(sum2[w], o);
                    }
#pragma unroll
                    for (int p = 0; p < P2; ++p) o[p] = dpp_mov<0xB1>(sum2[w][p]);
                    planes_add<P2, P2>(sum2[w], o);
#pragma unroll
                    for (int p = 0; p < P2; ++p) o[p] = dpp_mov<0x4E>(sum2[w][p]);
                    planes_add<P2, P2>(sum2[w], o);
                    // 65536 / L is a power of two: phi(S / (m L)) summed over the vectors = S << (16 - log2 L), below 2^32
                    // for documents shorter than 65536 vectors; the mean is that over m, rounded half up, 0 if m = 0
                    constexpr int SH = 16 - (P - 1);
                    static_assert((1 << (P - 1)) == L, "L is a power of two");
                    uint32_t part = 0;
#pragma unroll
                    for (int jq = 0; jq < 32 / G; ++jq) {
                        const uint32_t q = sub + G * jq;
                        uint32_t v = 0;
#pragma unroll
                        for (int p = P2 - 1; p >= 0; --p) v = 2 * v + ((sum2[w][p] >> q) & 1u);
                        uint32_t term = m ? ((v << SH) + m / 2) / m : 0u;
                        if (WEIGHTED && c0 + q < q_len[w])
                            term = (uint32_t)(((uint64_t)a.q_weights[q_lo[w] + c0 + q] * term + 32768) >> 16);
                        part += term;
                    }
                    if constexpr (G == 8) part += dpp_mov<0x141>(part);
                    part += dpp_mov<0xB1>(part);
                    part += dpp_mov<0x4E>(part);
                    score = (int32_t)part;
                }
                if (valid && sub == 0 && b0 + w < a.n_queries && c0 < q_len[w]) {
                    // W > 1 implies every set scores every document: set b0+w starts at (b0+w)*n_docs
                    int32_t* dst = a.scores + (W == 1 ? sp.base + meta.slot[doc] : (uint64_t)(b0 + w) * a.n_docs + first + doc);
                    if (W == 1 && m == 0 && meta.lo[doc] == ~0ull) {
                        if (c0 == 0) *dst = -1;  // empty candidate slot
                    } else if (SPLIT) {
                        if (score) atomicAdd(dst, score);
                    } else if (c0 == 0) {
                        *dst = score;
                    } else {
                        *dst += score;
                    }
                }
            }
        }
    }
}

// Stand-alone form of the candidate grouping (cand_order.hpp): one workgroup per list.
constexpr uint32_t ORDER_THREADS = 512, ORDER_MAX_RANGES = 4096;
__global__ __launch_bounds__(ORDER_THREADS) void cand_order_kernel(CandOrderArgs a) {
    __shared__ uint32_t bin[ORDER_MAX_RANGES];
    __shared__ uint32_t wave_sum[ORDER_THREADS / 64];
    cand_order_body<ORDER_THREADS>(a, blockIdx.x, bin, wave_sum);
}

uint64_t score_order_min() { return 1024; }

bool cand_order_plan(const uint32_t* cand_ids, const uint64_t* cand_off, uint64_t cand_uniform, uint32_t n_queries,
                     uint64_t max_scored, uint64_t n_docs, uint32_t max_ranges, uint32_t* order, CandOrderArgs* out) {
    if (n_queries == 0 || max_scored == 0 || max_scored > 0xFFFFFFFFull || max_ranges == 0) return false;  // slots are 32-bit
    uint32_t id_bits = 1;
    while (id_bits < 32 && ((n_docs ? n_docs - 1 : 0) >> id_bits)) ++id_bits;
    uint32_t log_ranges = 0;   // about 128 candidates per range when the ids are spread evenly
    while ((128ull << log_ranges) < max_scored && (2u << log_ranges) <= max_ranges && log_ranges < id_bits) ++log_ranges;
    *out = CandOrderArgs{cand_ids, cand_off, cand_uniform, n_queries, id_bits - log_ranges, 1u << log_ranges, order};
    return true;
}

hipError_t launch_cand_order(const CandOrderArgs& a, hipStream_t stream) {
    if (a.n_lists == 0) return hipSuccess;
    if (a.ranges > ORDER_MAX_RANGES) return hipErrorInvalidValue;
    hipLaunchKernelGGL(cand_order_kernel, dim3(a.n_lists), dim3(ORDER_THREADS), 0, stream, a);
    return hipGetLastError();
}

__global__ void fill_zero_kernel(int32_t* __restrict__ p, uint64_t n) {
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x)
        p[i] = 0;
}

static hipError_t launch_fill_zero(int32_t* p, uint64_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    uint64_t blocks = (n + 1023) / 1024;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, p, n);
    return hipGetLastError();
}

// A table of at most SCORE_TABLE_MAX words travels as a kernel argument and is written to device memory by the launch itself:
// in stream order behind the searches that still read the old table, with no staging buffer and no synchronisation.
struct ScoreTableArg {
    uint32_t v[SCORE_TABLE_MAX];
};
__global__ void write_table_kernel(ScoreTableArg t, uint32_t n, uint32_t* __restrict__ dst) {
    if (threadIdx.x < n) dst[threadIdx.x] = t.v[threadIdx.x];
}

hipError_t launch_write_table(const uint32_t* table_host, uint32_t n, uint32_t* dst, hipStream_t stream) {
    if (n > SCORE_TABLE_MAX || !dst) return hipErrorInvalidValue;
    ScoreTableArg arg{};
    for (uint32_t i = 0; i < n; ++i) arg.v[i] = table_host[i];
    hipLaunchKernelGGL(write_table_kernel, dim3(1), dim3(SCORE_TABLE_MAX), 0, stream, arg, n, dst);
    return hipGetLastError();
}

__global__ void reset_first_bad_kernel(unsigned long long* first_bad) { *first_bad = ~0ull; }

__global__ __launch_bounds__(256) void check_cand_ids_kernel(const uint32_t* __restrict__ ids, uint64_t n, uint64_t n_docs,
                                                             unsigned long long* first_bad) {
    unsigned long long worst = ~0ull;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t id = ids[i];
        if (id != 0xFFFFFFFFu && id >= n_docs && i < worst) worst = i;
    }
    if (worst != ~0ull) atomicMin(first_bad, worst);
}

hipError_t launch_check_cand_ids(const uint32_t* cand_ids, uint64_t n, uint64_t n_docs, unsigned long long* first_bad,
                                 hipStream_t stream) {
    if (!first_bad) return hipErrorInvalidValue;
    hipLaunchKernelGGL(reset_first_bad_kernel, dim3(1), dim3(1), 0, stream, first_bad);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n == 0) return e;
    uint64_t blocks = (n + 2047) / 2048;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(check_cand_ids_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, cand_ids, n, n_docs, first_bad);
    return hipGetLastError();
}

// One-byte codes: L in {8, 16, 32, 64, 128}.  16-bit codes: the L * 2^C * 4-byte table has to fit 64 KB of LDS.
bool score_masklut_supported(uint32_t L, uint32_t C) {
    if (C >= 1 && C <= 8) return L == 8 || L == 16 || L == 32 || L == 64 || L == 128;
    return (L == 8 && C <= 11) || (L == 16 && C <= 10) || (L == 32 && C == 9);
}

template <int L, int CB, int CW>
static hipError_t launch_masklut_t(const ScoreArgs& a, hipStream_t stream, char* desc, size_t desc_len) {
    // two query sets per workgroup when every document is scored for every set and the paired table (8 bytes per entry)
    // is at most 32 KB, or 64 KB with at most 32 tables (512 threads share it then; the offsets still fit the 16-bit
    // immediate of an LDS read).  With one set per workgroup those shapes are bound by LDS: half the arithmetic per read.
    constexpr size_t PAIR_BYTES = (size_t)L * (1u << CB) * 8;
    constexpr bool PAIR_OK = PAIR_BYTES <= 32 * 1024 || (L <= 32 && PAIR_BYTES <= 64 * 1024);
    bool pair = PAIR_OK && a.cand_ids == nullptr && a.n_queries >= 2 && !a.sigma_mean;  // the mean form takes one set per workgroup
    // documents per workgroup: at most LUT_DOCS; fewer when that would leave the 256 CUs short of
    // workgroups, but at least 64 (32 = one run of 8 documents for each of the four waves when the
    // documents are long: about 4096 vectors per workgroup keep the table build amortised)
    uint32_t gy = pair ? (a.n_queries + 1) / 2 : a.n_queries;
    const uint64_t mean_len = a.n_docs ? (a.n_vectors + a.n_docs - 1) / a.n_docs : 1;
    const uint32_t wave_docs = masklut_threads(L, CB, CW, pair ? 2 : 1) / 64 * 8;  // one run of 8 documents per wave
    uint32_t dpb_min = wave_docs > 64 ? wave_docs : 64;
    while (dpb_min > wave_docs && (uint64_t)(dpb_min / 2) * mean_len >= 4096) dpb_min /= 2;
    // a single short list (one query set's candidates): even 64 documents per workgroup leave most CUs idle and the launch
    // is a chain of memory round trips per workgroup, so one run of documents per wave
    if (((a.max_scored + 63) / 64) * gy < 256) dpb_min = wave_docs;
    // candidate lists are gathered from all over the code array and the kernel is bound by those reads:
    // smaller workgroups (their start-up phases overlap better) measure faster as long as the table is small
    uint32_t dpb = (a.cand_ids && (size_t)L * (1u << CB) * 4 <= 16 * 1024) ? LUT_DOCS / 2 : LUT_DOCS;
    while (dpb > dpb_min && ((a.max_scored + dpb - 1) / dpb) * gy < 4096) dpb /= 2;
    uint64_t bx = (a.max_scored + dpb - 1) / dpb;
    if (bx > 0x7fffffffull || a.n_queries > 65535) return hipErrorInvalidValue;
    // long query sets on a grid that is still small: split the 32-vector chunks over gz workgroups
    const uint32_t chunks = (a.max_q_len + 31) / 32;
    uint32_t gz = 1;
    if (chunks > 1 && bx * gy < 2048) {
        pair = false;  // the split kernels take one query set per workgroup
        gy = a.n_queries;
        gz = (uint32_t)((2048 + bx * gy - 1) / (bx * gy));
        if (gz > chunks) gz = chunks;
        if (gz < 2) gz = 2;
    }
    const uint64_t gyz = (uint64_t)gy * gz;
    if (gyz > 65535) return hipErrorInvalidValue;
    if (gz > 1) {  // partial sums are added into the scores
        const uint64_t n = a.cand_ids ? a.total_scored : (uint64_t)a.n_queries * a.n_docs;
        hipError_t e = launch_fill_zero(a.scores, n, stream);
        if (e != hipSuccess) return e;
    }
    // exhaustive mode, and candidate lists ordered by id range: linear grid with the XCD-aware decode (document
    // blocks rounded up to 8), so that the workgroups of one block of positions run back to back for all query sets
    dim3 grid((unsigned)bx, (unsigned)gyz);
    uint32_t gy_linear = 0;
    if (a.cand_ids == nullptr || a.order != nullptr) {
        const uint64_t total = (bx + 7) / 8 * 8 * gyz;
        if (total <= 0x7fffffffull) {
            grid = dim3((unsigned)total);
            gy_linear = (uint32_t)gyz;
        }
    }
    // transform form of the kernel: raw counts, tabulated phi of the maximum (weighted or not), mean of the counts
    const int remap = a.sigma_mean ? (a.q_weights ? 4 : 3) : a.q_weights ? 2 : a.remap ? 1 : 0;
    // the instantiation as a profiler prints it
    if (desc)
        snprintf(desc, desc_len, "score_masklut_kernel<%d, %d, %d, %d, %d, %s>", L, CB, CW, remap, pair ? 2 : 1,
                 gz > 1 ? "true" : "false");
    using Kernel = void (*)(ScoreArgs, uint32_t, uint32_t, uint32_t);
    if constexpr (PAIR_OK) {
        if (pair) {
            const Kernel kern2 = remap == 2   ? score_masklut_kernel<L, CB, CW, 2, 2, false>
                                 : remap == 1 ? score_masklut_kernel<L, CB, CW, 1, 2, false>
                                              : score_masklut_kernel<L, CB, CW, 0, 2, false>;
            hipLaunchKernelGGL(kern2, grid, dim3(masklut_threads(L, CB, CW, 2)), 0, stream, a, dpb, gy_linear, 1u);
            return hipGetLastError();
        }
    }
    Kernel kern;
    if (gz > 1)
        kern = remap == 4   ? score_masklut_kernel<L, CB, CW, 4, 1, true>
               : remap == 3 ? score_masklut_kernel<L, CB, CW, 3, 1, true>
               : remap == 2 ? score_masklut_kernel<L, CB, CW, 2, 1, true>
               : remap == 1 ? score_masklut_kernel<L, CB, CW, 1, 1, true>
                            : score_masklut_kernel<L, CB, CW, 0, 1, true>;
    else
        kern = remap == 4   ? score_masklut_kernel<L, CB, CW, 4, 1, false>
               : remap == 3 ? score_masklut_kernel<L, CB, CW, 3, 1, false>
               : remap == 2 ? score_masklut_kernel<L, CB, CW, 2, 1, false>
               : remap == 1 ? score_masklut_kernel<L, CB, CW, 1, 1, false>
                            : score_masklut_kernel<L, CB, CW, 0, 1, false>;
    hipLaunchKernelGGL(kern, grid, dim3(masklut_threads(L, CB, CW, 1)), 0, stream, a, dpb, gy_linear, gz);
    return hipGetLastError();
}

hipError_t launch_score_masklut(const ScoreArgs& a, hipStream_t stream, char* desc, size_t desc_len) {
    if (desc && desc_len) desc[0] = 0;
    if (a.n_queries == 0 || a.max_scored == 0) return hipSuccess;
    if (!score_masklut_supported(a.L, a.C) || a.code_bytes != (a.C > 8 ? 2u : 1u)) return hipErrorInvalidValue;
    // a tabulated phi of the maximum, or the mean of the counts themselves (phi = identity)
    if ((a.sigma_mean && !a.phi_identity) || (a.q_weights && !a.remap)) return hipErrorInvalidValue;
    const uint32_t cb = a.C <= 6 ? 6 : a.C;
#define DESSERT_LUT_CASE(L_, CB_, CW_) \
    if (a.L == L_ && cb == CB_) return launch_masklut_t<L_, CB_, CW_>(a, stream, desc, desc_len);
    DESSERT_LUT_CASE(8, 6, 1) DESSERT_LUT_CASE(8, 7, 1) DESSERT_LUT_CASE(8, 8, 1)
    DESSERT_LUT_CASE(16, 6, 1) DESSERT_LUT_CASE(16, 7, 1) DESSERT_LUT_CASE(16, 8, 1)
    DESSERT_LUT_CASE(32, 6, 1) DESSERT_LUT_CASE(32, 7, 1) DESSERT_LUT_CASE(32, 8, 1)
    DESSERT_LUT_CASE(64, 6, 1) DESSERT_LUT_CASE(64, 7, 1) DESSERT_LUT_CASE(64, 8, 1)
    DESSERT_LUT_CASE(128, 6, 1) DESSERT_LUT_CASE(128, 7, 1) DESSERT_LUT_CASE(128, 8, 1)
    DESSERT_LUT_CASE(8, 9, 2) DESSERT_LUT_CASE(8, 10, 2) DESSERT_LUT_CASE(8, 11, 2)
    DESSERT_LUT_CASE(16, 9, 2) DESSERT_LUT_CASE(16, 10, 2)
    DESSERT_LUT_CASE(32, 9, 2)
#undef DESSERT_LUT_CASE
    return hipErrorInvalidValue;
}

}  // namespace dessert
