/* Host-side paths of the C ABI that run without a GPU, for a build whose host code is instrumented with
 * AddressSanitizer and UndefinedBehaviorSanitizer (tests/test_host_sanitized.py): configuration checks of
 * dessert_create, NULL handles and NULL arguments of every entry point, the message buffer.  Every call must come
 * back with a status; the sanitizers abort the process on any bad access or undefined operation. */
#include <stdio.h>
#include <string.h>

#include "../../include/dessert.h"

static int failures = 0;
#define EXPECT(cond)                                                        \
    do {                                                                    \
        if (!(cond)) {                                                      \
            printf("FAILED line %d: %s  (last error: %s)\n", __LINE__, #cond, dessert_last_error()); \
            ++failures;                                                     \
        }                                                                   \
    } while (0)

int main(void) {
    dessert_index_t *ix = (dessert_index_t *)0x1;
    dessert_config_t c;
    memset(&c, 0, sizeof c);
    c.d = 128; c.L = 32; c.C = 7; c.dtype = DESSERT_I8; c.proj_kind = DESSERT_PROJ_RADEMACHER_I8; c.seed = 1;

    /* configuration errors are found before any device is touched */
    EXPECT(dessert_create(NULL, &ix) == DESSERT_EINVAL);
    EXPECT(dessert_create(&c, NULL) == DESSERT_EINVAL);
    dessert_config_t b = c;
    b.d = 0;  EXPECT(dessert_create(&b, &ix) == DESSERT_EINVAL && ix == NULL);
    b = c; b.C = 0;   EXPECT(dessert_create(&b, &ix) == DESSERT_EINVAL);
    b = c; b.C = 17;  EXPECT(dessert_create(&b, &ix) == DESSERT_EINVAL && strstr(dessert_last_error(), "C must be"));
    b = c; b.L = 3;   EXPECT(dessert_create(&b, &ix) == DESSERT_EINVAL);
    b = c; b.L = 132; EXPECT(dessert_create(&b, &ix) == DESSERT_EINVAL && strstr(dessert_last_error(), "L must be"));
    b = c; b.L = 30;  EXPECT(dessert_create(&b, &ix) == DESSERT_EINVAL);
    b = c; b.dtype = 7;     EXPECT(dessert_create(&b, &ix) == DESSERT_EINVAL);
    b = c; b.proj_kind = 9; EXPECT(dessert_create(&b, &ix) == DESSERT_EINVAL);
    b = c; b.proj_kind = DESSERT_PROJ_GAUSSIAN_F32; EXPECT(dessert_create(&b, &ix) == DESSERT_EINVAL);
    b = c; b.d = 1u << 30; b.L = 128; b.C = 16; EXPECT(dessert_create(&b, &ix) == DESSERT_EINVAL);
    /* a valid configuration: no device here, so a loud failure (or a handle, on a machine with a GPU) */
    dessert_status_t st = dessert_create(&c, &ix);
    EXPECT(st == DESSERT_EHIP || st == DESSERT_OK || st == DESSERT_EINVAL);
    if (st == DESSERT_OK) { dessert_destroy(ix); ix = NULL; }
    else EXPECT(ix == NULL && strlen(dessert_last_error()) > 0);

    /* NULL handles and arguments */
    float ms[4];
    uint32_t len = 1;
    uint64_t off[2] = {0, 1};
    dessert_destroy(NULL);
    EXPECT(dessert_get_projection(NULL, &c) == DESSERT_EINVAL);
    EXPECT(dessert_set_algo(NULL, 0, 0) == DESSERT_EINVAL);
    EXPECT(dessert_set_score_transform(NULL, 1) == DESSERT_EINVAL);
    EXPECT(dessert_set_query_weights(NULL, NULL, 0) == DESSERT_EINVAL);
    EXPECT(dessert_set_debug(NULL, 1) == DESSERT_EINVAL);
    EXPECT(dessert_code_bytes(NULL, 10) == 0);
    EXPECT(dessert_hash(NULL, &c, 1, (uint8_t *)&c) == DESSERT_EINVAL);
    EXPECT(dessert_build_index(NULL, &c, 1, &len, 1, (uint8_t *)&c, off) == DESSERT_EINVAL);
    EXPECT(dessert_attach_index(NULL, (const uint8_t *)&c, off, 1, 1, 1) == DESSERT_EINVAL);
    EXPECT(dessert_search_workspace_bytes(NULL, 1, 1, 1, 1) == 0);
    EXPECT(dessert_search(NULL, &c, &len, 1, NULL, NULL, 0, &c, 256, &len, (int32_t *)&len) == DESSERT_EINVAL);
    EXPECT(dessert_search(NULL, &c, &len, 1, NULL, NULL, 5, &c, 256, NULL, NULL) == DESSERT_EINVAL);
    EXPECT(dessert_search(NULL, &c, &len, 1, NULL, NULL, 5, &c, 256, &len, (int32_t *)&len) == DESSERT_EINVAL);
    EXPECT(dessert_scores(NULL, &c, &len, 1, NULL, NULL, &c, 256, NULL) == DESSERT_EINVAL);
    EXPECT(dessert_scores(NULL, &c, &len, 1, NULL, NULL, &c, 256, (int32_t *)&len) == DESSERT_EINVAL);
    EXPECT(dessert_noalloc_scratch_bytes() == DESSERT_NOALLOC_SCRATCH_BYTES);
    EXPECT(dessert_search_noalloc(NULL, &c, 1, 1, NULL, 0, 5, &len, (int32_t *)&len) == DESSERT_EINVAL);
    EXPECT(dessert_search_noalloc(NULL, &c, 1, 1, NULL, 0, 0, &len, (int32_t *)&len) == DESSERT_EINVAL);
    EXPECT(dessert_filter_kmeans_workspace_bytes(NULL, 1, 1) == 0);
    EXPECT(dessert_filter_kmeans(NULL, (const int8_t *)&c, 1, (int8_t *)&c, 1, 1, &c, 256) == DESSERT_EINVAL);
    EXPECT(dessert_filter_build(NULL, (const int8_t *)&c, 1, &c, &len, &len, &len) == DESSERT_EINVAL);
    EXPECT(dessert_filter_workspace_bytes(NULL, 1, 1, 1, 1) == 0);
    EXPECT(dessert_filter_query(NULL, &c, &len, 1, 1, 1, &c, 256, &len, (int32_t *)&len) == DESSERT_EINVAL);
    EXPECT(dessert_filter_search_workspace_bytes(NULL, 1, 1, 1, 1, 1, 1) == 0);
    EXPECT(dessert_filter_search(NULL, &c, &len, 1, 1, 1, 1, &c, 256, &len, (int32_t *)&len) == DESSERT_EINVAL);
    EXPECT(dessert_enable_timing(NULL, 1) == DESSERT_EINVAL);
    EXPECT(dessert_get_timing(NULL, 0, ms) == DESSERT_EINVAL);
    EXPECT(strcmp(dessert_last_score_kernel(NULL), "") == 0);
    EXPECT(dessert_probe_read_bandwidth(NULL, 0, 0, NULL, 1, ms) == DESSERT_EINVAL);
    EXPECT(dessert_probe_read_bandwidth(&c, 8, 0, NULL, 1, ms) == DESSERT_EINVAL);
    EXPECT(dessert_probe_mix_bandwidth(NULL, NULL, 0, 0, NULL, 1, ms) == DESSERT_EINVAL);
    EXPECT(strlen(dessert_version()) > 0);
    EXPECT(strlen(dessert_last_error()) < 512);

    if (failures) return 1;
    printf("C ABI host sanitizer run: ok\n");
    return 0;
}
