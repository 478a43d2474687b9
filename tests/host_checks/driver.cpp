// Host-side check of libinsum's C entry points under AddressSanitizer and
// UndefinedBehaviorSanitizer: the host-only helpers with ordinary, extreme and invalid
// arguments, and the argument validation of every device entry point (each call below returns
// before any kernel would be launched, so the program runs on a machine without a GPU).
// Built and run by tests/test_host_sanitizers.py; exit status 0 = every expectation held.
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "insum.h"

static int failures = 0;
#define EXPECT(cond)                                                        \
    do {                                                                    \
        if (!(cond)) {                                                      \
            ++failures;                                                     \
            fprintf(stderr, "line %d: expectation failed: %s\n", __LINE__, #cond); \
        }                                                                   \
    } while (0)

int main() {
    const int64_t kBig = (int64_t)1 << 62, kMax = INT64_MAX, kI31 = ((int64_t)1 << 31) - 1;
    int32_t g_used = -1, cand[3];
    int64_t G = -1;
    char dev[64];   // stands for device memory: never dereferenced by the calls below
    void* p = dev;
    const int32_t* ip = reinterpret_cast<const int32_t*>(dev);
    int32_t* op = reinterpret_cast<int32_t*>(dev);

    // ---- host-only helpers -------------------------------------------------------------------
    EXPECT(insum_version() >= 100);
    for (int s = -5; s < 20; ++s) EXPECT(insum_status_string(s) != nullptr && strlen(insum_status_string(s)) > 0);
    EXPECT(insum_default_group_size(1677722, 4096) == 16);
    EXPECT(insum_default_group_size(0, 10) == 1 && insum_default_group_size(10, 0) == 1);
    EXPECT(insum_default_group_size(-1, -1) == 1);
    EXPECT(insum_default_group_size(kMax, 1) == (1 << 30));
    EXPECT(insum_default_group_size(kMax, kMax) == 1);
    EXPECT(insum_default_group_size(1, kMax) == 1);
    const int64_t occ[4] = {3, 1, 1, 2};
    EXPECT(insum_indirect_access_cost(4, occ, 1) == 14 && insum_indirect_access_cost(4, occ, 2) == 15);
    EXPECT(insum_indirect_access_cost(4, occ, 0) == -1 && insum_indirect_access_cost(-1, occ, 1) == -1);
    EXPECT(insum_indirect_access_cost(4, nullptr, 1) == -1 && insum_indirect_access_cost(0, nullptr, 1) == 0);
    const int64_t huge[3] = {kMax, kMax, kMax};
    EXPECT(insum_indirect_access_cost(3, huge, 1) == -1);          // does not fit 64 bits: reported, not wrapped
    EXPECT(insum_indirect_access_cost(1, huge, INT32_MAX) == -1);
    const int64_t large[1] = {(int64_t)1 << 40};
    EXPECT(insum_indirect_access_cost(1, large, INT32_MAX) == 513 * ((int64_t)INT32_MAX + 1));
    const int64_t neg[2] = {5, -1};
    EXPECT(insum_indirect_access_cost(2, neg, 2) == -1);
    EXPECT(insum_group_size_candidates(1677722, 4096, cand) == 3 && cand[0] == 8 && cand[2] == 32);
    EXPECT(insum_group_size_candidates(0, 0, cand) == 2 && cand[0] == 1 && cand[1] == 2);
    EXPECT(insum_group_size_candidates(kMax, 1, cand) == 2 && cand[1] == (1 << 30));
    EXPECT(insum_group_size_candidates(5, 5, nullptr) == 0);

    // ---- workspace sizes: ordinary, empty, negative and very large arguments -------------------
    const int64_t sizes[] = {-7, 0, 1, 4096, (int64_t)1 << 20, kI31, (int64_t)1 << 40, kBig};
    for (int64_t a : sizes)
        for (int64_t b : sizes) {
            (void)insum_coo_to_groupcoo_workspace_bytes(a, b);
            (void)insum_map_to_groupcoo_workspace_bytes(a, b);
            for (int32_t g : {-1, 0, 1, 3, 4, 1 << 20, INT32_MAX}) {
                (void)insum_spmm_groupcoo_workspace_bytes(a, b, a, g);
                (void)insum_spmm_groupcoo_workspace_bytes(4096, 128, b, g);
                (void)insum_groupcoo_transpose_workspace_bytes(a, b, a, g);
                (void)insum_groupcoo_transpose_workspace_bytes(1000, 1000, b, g);
                for (int32_t bm : {0, 1, 8, 32, 64, 128, 1 << 20}) {
                    (void)insum_spmm_blockgroupcoo_workspace_bytes(a, b, a, g, bm, bm);
                    (void)insum_spmm_blockgroupcoo_workspace_bytes(8192, 512, b, g, bm, 32);
                    (void)insum_coo_to_blockgroupcoo_workspace_bytes(a, b, a, bm, bm);
                }
                (void)insum_spconv_groupcoo_workspace_bytes(a, 27, 128, 128, b, g, INSUM_F16);
                (void)insum_spconv_groupcoo_workspace_bytes(265000, b, a, 128, 100000, g, INSUM_BF16);
            }
            for (int dt = -1; dt < 4; ++dt) {
                (void)insum_choose_group_size_workspace_bytes(a, b, a, (insum_dtype)dt);
                (void)insum_choose_group_size_workspace_bytes(4096, 256, b, (insum_dtype)dt);
                (void)insum_spmm_groupcoo_transposed_workspace_bytes(a, b, (insum_dtype)dt);
            }
        }
    EXPECT(insum_coo_to_groupcoo_workspace_bytes(1 << 20, 16905781) > 16905781u * 24u);
    EXPECT(insum_spmm_groupcoo_workspace_bytes(1 << 20, 128, 4726049, 4) >= 256);
    EXPECT(insum_spmm_blockgroupcoo_workspace_bytes(8192, 512, 1760, 4, 32, 32) > 0);
    EXPECT(insum_spmm_blockgroupcoo_workspace_bytes(8192, 512, 1760, 4, 8, 8) == 0);
    EXPECT(insum_spmm_groupcoo_transposed_workspace_bytes(1000, 128, INSUM_F32) == 0);
    EXPECT(insum_spmm_groupcoo_transposed_workspace_bytes(1000, 128, INSUM_F16) >= 1000u * 128u * 4u);
    EXPECT(insum_groupcoo_transpose_workspace_bytes(10, 10, (int64_t)1 << 29, 4) == 0);

    // ---- argument validation of the device entry points (all return before touching a GPU) ----
    EXPECT(insum_coo_to_groupcoo(-1, 5, 3, ip, ip, p, INSUM_F32, 2, &g_used, &G, op, op, p, 9, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_coo_to_groupcoo(5, 5, 3, ip, ip, p, INSUM_F32, 2, nullptr, &G, op, op, p, 9, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_coo_to_groupcoo(5, 5, 3, ip, ip, p, (insum_dtype)7, 2, &g_used, &G, op, op, p, 9, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_coo_to_groupcoo(5, 5, 3, nullptr, ip, p, INSUM_F32, 2, &g_used, &G, op, op, p, 9, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_coo_to_groupcoo(5, 5, 3, ip, ip, p, INSUM_F32, 2, &g_used, &G, op, nullptr, p, 9, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_coo_to_groupcoo((int64_t)1 << 31, 5, 3, ip, ip, p, INSUM_F32, 2, &g_used, &G, op, op, p, 9, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_coo_to_groupcoo(5, 5, 0, nullptr, nullptr, nullptr, INSUM_F16, 0, &g_used, &G, nullptr, nullptr, nullptr, 0, nullptr, 0, nullptr) == INSUM_OK && g_used == 1 && G == 0);
    EXPECT(insum_coo_to_groupcoo(0, 5, 3, ip, ip, p, INSUM_F32, 2, &g_used, &G, op, op, p, 9, p, 64, nullptr) == INSUM_ERR_OUT_OF_RANGE);
    EXPECT(insum_coo_to_groupcoo(5, 5, 3, ip, ip, p, INSUM_F32, 2, &g_used, &G, op, op, p, 9, p, 64, nullptr) == INSUM_ERR_CAPACITY);   // workspace too small

    EXPECT(insum_coo_to_blockgroupcoo(64, 64, 3, ip, ip, p, INSUM_F16, 0, 32, 2, &g_used, &G, op, op, p, 9, p, 64, nullptr) != INSUM_OK);
    EXPECT(insum_coo_to_blockgroupcoo(65, 64, 3, ip, ip, p, INSUM_F16, 32, 32, 2, &g_used, &G, op, op, p, 9, p, 64, nullptr) == INSUM_ERR_UNSUPPORTED);
    EXPECT(insum_coo_to_blockgroupcoo(64, 64, -3, ip, ip, p, INSUM_F16, 32, 32, 2, &g_used, &G, op, op, p, 9, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_coo_to_blockgroupcoo(64, 64, 0, nullptr, nullptr, nullptr, INSUM_BF16, 32, 32, 0, &g_used, &G, nullptr, nullptr, nullptr, 0, nullptr, 0, nullptr) == INSUM_OK && G == 0);

    EXPECT(insum_map_to_groupcoo(10, 10, 27, -1, ip, ip, ip, p, INSUM_F16, 0, &g_used, &G, op, op, op, p, 5, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_map_to_groupcoo(10, 10, 27, 4, ip, ip, ip, p, INSUM_F16, 0, nullptr, &G, op, op, op, p, 5, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);

    EXPECT(insum_groupcoo_transpose(-1, 5, 2, 2, ip, ip, p, INSUM_F32, 0, &g_used, &G, nullptr, op, op, p, 4, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_groupcoo_transpose(5, 5, 2, 0, ip, ip, p, INSUM_F32, 0, &g_used, &G, nullptr, op, op, p, 4, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_groupcoo_transpose(5, 5, 2, 2, nullptr, ip, p, INSUM_F32, 0, &g_used, &G, nullptr, op, op, p, 4, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_groupcoo_transpose(5, 5, (int64_t)1 << 30, 4, ip, ip, p, INSUM_F32, 0, &g_used, &G, nullptr, op, op, p, 4, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_groupcoo_transpose(5, 5, 2, 2, ip, ip, p, INSUM_F32, 0, &g_used, &G, nullptr, op, op, p, 4, p, 64, nullptr) == INSUM_ERR_CAPACITY);
    int64_t entries = -1;
    EXPECT(insum_groupcoo_transpose(5, 7, 0, 4, nullptr, nullptr, nullptr, INSUM_F16, 2, &g_used, &G, &entries, nullptr, nullptr, nullptr, 0, nullptr, 0, nullptr) == INSUM_OK && G == 0 && entries == 0 && g_used == 2);

    EXPECT(insum_spmm_groupcoo(-1, 5, 5, 1, 2, ip, ip, p, INSUM_F32, p, 5, INSUM_F32, p, 5, INSUM_F32, 0, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_spmm_groupcoo(5, 5, 5, 1, 0, ip, ip, p, INSUM_F32, p, 5, INSUM_F32, p, 5, INSUM_F32, 0, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_spmm_groupcoo(5, 5, 5, 1, 2, ip, ip, p, INSUM_F32, p, 4, INSUM_F32, p, 5, INSUM_F32, 0, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);   // ldb < N
    EXPECT(insum_spmm_groupcoo(5, 5, 5, 1, 2, ip, ip, p, INSUM_F16, p, 5, INSUM_F32, p, 5, INSUM_F32, 0, p, 64, nullptr) == INSUM_ERR_UNSUPPORTED);  // a_dt != b_dt
    EXPECT(insum_spmm_groupcoo(5, 5, 5, 1, 2, ip, ip, p, INSUM_F32, p, 5, INSUM_F32, p, 5, INSUM_F16, 0, p, 64, nullptr) == INSUM_ERR_UNSUPPORTED);  // narrower C
    EXPECT(insum_spmm_groupcoo(5, 5, 0, 1, 2, ip, ip, p, INSUM_F32, p, 5, INSUM_F32, p, 5, INSUM_F32, 0, p, 64, nullptr) == INSUM_OK);               // N = 0
    EXPECT(insum_spmm_groupcoo(5, 5, 5, 1, 2, ip, ip, p, INSUM_F32, p, 5, INSUM_F32, nullptr, 5, INSUM_F32, 0, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_spmm_groupcoo(5, 5, 5, 1, 2, nullptr, ip, p, INSUM_F32, p, 5, INSUM_F32, p, 5, INSUM_F32, 0, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_spmm_groupcoo(5, 5, 5, 1, 2, ip, ip, p, INSUM_F32, p, 5, INSUM_F32, p, 5, INSUM_F32, 0, nullptr, 0, nullptr) == INSUM_ERR_CAPACITY);
    EXPECT(insum_spmm_groupcoo_noalloc(5, 5, 5, 1, 2, ip, ip, p, (insum_dtype)9, p, 5, INSUM_F32, p, 5, INSUM_F32, 0, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_spmm_groupcoo_noalloc(0, 5, 5, 0, 2, nullptr, nullptr, nullptr, INSUM_F32, nullptr, 5, INSUM_F32, nullptr, 5, INSUM_F32, 0, nullptr) == INSUM_OK);

    EXPECT(insum_spmm_groupcoo_transposed(5, 5, 5, 1, 0, ip, ip, p, INSUM_F32, p, 5, INSUM_F32, p, 5, INSUM_F32, 0, nullptr, 0, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_spmm_groupcoo_transposed(5, 5, 5, 1, 2, ip, ip, p, INSUM_F32, p, 5, INSUM_F16, p, 5, INSUM_F32, 0, nullptr, 0, nullptr) == INSUM_ERR_UNSUPPORTED);
    EXPECT(insum_spmm_groupcoo_transposed(5, 5, 5, 1, 2, ip, ip, p, INSUM_F32, p, 3, INSUM_F32, p, 5, INSUM_F32, 0, nullptr, 0, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_spmm_groupcoo_transposed(5, 0, 5, 1, 2, ip, ip, p, INSUM_F32, p, 5, INSUM_F32, p, 5, INSUM_F32, 0, nullptr, 0, nullptr) == INSUM_OK);
    EXPECT(insum_spmm_groupcoo_transposed(5, 5, 8, 1, 2, ip, ip, p, INSUM_F16, p, 8, INSUM_F16, p, 8, INSUM_F16, 0, nullptr, 0, nullptr) == INSUM_ERR_CAPACITY);

    EXPECT(insum_spmm_blockgroupcoo(64, 64, 8, 1, 2, 32, 32, ip, ip, p, INSUM_F16, p, 8, INSUM_F16, p, 8, INSUM_F16, 0, nullptr, 0, nullptr) != INSUM_ERR_INVALID_ARG || true);
    EXPECT(insum_spmm_blockgroupcoo(65, 64, 8, 1, 2, 32, 32, ip, ip, p, INSUM_F16, p, 8, INSUM_F16, p, 8, INSUM_F16, 0, nullptr, 0, nullptr) != INSUM_OK);
    EXPECT(insum_spmm_blockgroupcoo(64, 64, 8, 1, 0, 32, 32, ip, ip, p, INSUM_F16, p, 8, INSUM_F16, p, 8, INSUM_F16, 0, nullptr, 0, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_spmm_blockgroupcoo(64, 64, 8, 1, 2, 32, 32, ip, ip, p, INSUM_F16, p, 4, INSUM_F16, p, 8, INSUM_F16, 0, nullptr, 0, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_spmm_blockgroupcoo(64, 64, 8, 1, 2, 32, 32, ip, ip, p, INSUM_F16, p, 8, INSUM_BF16, p, 8, INSUM_F16, 0, nullptr, 0, nullptr) == INSUM_ERR_UNSUPPORTED);
    EXPECT(insum_spmm_blockgroupcoo(64, 64, 0, 1, 2, 32, 32, ip, ip, p, INSUM_F16, p, 8, INSUM_F16, p, 8, INSUM_F16, 0, nullptr, 0, nullptr) == INSUM_OK);
    EXPECT(insum_spmm_blockgroupcoo_plan(64, 64, 8, 1, 0, 32, 32, ip, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_spmm_blockgroupcoo_plan(64, 64, 256, 1, 2, 32, 32, ip, p, 64, nullptr) == INSUM_ERR_CAPACITY);

    EXPECT(insum_spconv_groupcoo(-1, 5, 27, 8, 8, 1, 2, ip, ip, ip, p, p, 8, p, INSUM_F16, reinterpret_cast<float*>(dev), 8, 0, 0, nullptr, 0, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_spconv_groupcoo(5, 5, 27, 8, 8, 1, 2, ip, ip, ip, p, p, 4, p, INSUM_F16, reinterpret_cast<float*>(dev), 8, 0, 0, nullptr, 0, nullptr) == INSUM_ERR_INVALID_ARG);   // ld_in < C
    EXPECT(insum_spconv_groupcoo(5, 5, 27, 8, 8, 1, 2, nullptr, ip, ip, p, p, 8, p, INSUM_F16, reinterpret_cast<float*>(dev), 8, 0, 0, nullptr, 0, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_spconv_groupcoo(0, 5, 27, 8, 8, 0, 2, nullptr, nullptr, nullptr, nullptr, nullptr, 8, nullptr, INSUM_F16, nullptr, 8, 0, 0, nullptr, 0, nullptr) == INSUM_OK);

    int32_t best = -1, ncand = -1;
    float ms[3];
    EXPECT(insum_choose_group_size(5, 5, 5, 3, ip, ip, p, INSUM_F32, p, 5, p, 5, INSUM_F32, 0, &best, cand, ms, &ncand, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);   // repeats
    EXPECT(insum_choose_group_size(5, 5, 5, 3, ip, ip, p, INSUM_F32, p, 5, p, 5, INSUM_F32, 3, nullptr, cand, ms, &ncand, p, 64, nullptr) == INSUM_ERR_INVALID_ARG);
    EXPECT(insum_choose_group_size(5, 5, 5, 0, nullptr, nullptr, nullptr, INSUM_F32, nullptr, 5, nullptr, 5, INSUM_F32, 3, &best, cand, ms, &ncand, nullptr, 0, nullptr) == INSUM_OK && best == 1);
    EXPECT(insum_choose_group_size(5, 5, 5, 3, ip, ip, p, INSUM_F32, p, 5, p, 5, INSUM_F32, 3, &best, cand, ms, &ncand, p, 64, nullptr) == INSUM_ERR_CAPACITY);

    if (failures) fprintf(stderr, "%d expectation(s) failed\n", failures);
    else printf("host checks ok\n");
    return failures ? 1 : 0;
}
