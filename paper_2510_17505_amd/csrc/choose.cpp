// Group size by measurement (Section 4.2, last paragraph: round g* = sqrt(S/n) to the nearest
// powers of two and keep the one that runs best).  Host code only: it drives the library's own
// conversion and SpMM entry points on the caller's stream and times them with HIP events.
#include <algorithm>

#include "common.h"

using namespace insum;

namespace {

struct Carve {
    uintptr_t cur, end;
    bool ok = true;
    Carve(void* base, size_t bytes)
        : cur((reinterpret_cast<uintptr_t>(base) + 255) / 256 * 256), end(reinterpret_cast<uintptr_t>(base) + bytes) {
        if (!base || cur > end) ok = false;
    }
    void* take(size_t bytes) {
        bytes = align_up(std::max<size_t>(bytes, 1), 256);
        if (!ok || cur + bytes > end) {
            ok = false;
            return nullptr;
        }
        void* p = reinterpret_cast<void*>(cur);
        cur += bytes;
        return p;
    }
};

int64_t group_capacity(int64_t M, int64_t nnz, int32_t g) { return nnz / g + std::min(M, nnz); }

}  // namespace

// The default of insum_default_group_size and its two power-of-two neighbours, ascending and
// without repetition: whichever side of the default g* lies on, the set holds both powers of
// two that enclose g*.
extern "C" int32_t insum_group_size_candidates(int64_t S, int64_t n, int32_t* out3) {
    if (!out3) return 0;
    const int32_t g0 = insum_default_group_size(S, n);
    int32_t count = 0;
    if (g0 >= 2) out3[count++] = g0 / 2;
    out3[count++] = g0;
    if (g0 <= (1 << 29)) out3[count++] = g0 * 2;
    return count;
}

extern "C" size_t insum_choose_group_size_workspace_bytes(int64_t M, int64_t N, int64_t nnz, insum_dtype dt) {
    if (M < 0 || N < 0 || nnz < 0 || !dtype_valid(dt)) return 0;
    if (M >= (1LL << 31) || N >= (1LL << 31) || nnz >= (1LL << 31)) return 0;   // beyond what the conversion accepts
    int32_t cand[3];
    const int32_t nc = insum_group_size_candidates(nnz, M, cand);
    size_t conv = insum_coo_to_groupcoo_workspace_bytes(M, nnz), spmm = 0, am = 0, ak = 0;
    for (int32_t i = 0; i < nc; ++i) {
        const int64_t cap = group_capacity(M, nnz, cand[i]);
        spmm = std::max(spmm, insum_spmm_groupcoo_workspace_bytes(M, N, cap, cand[i]));
        am = std::max(am, (size_t)cap * 4);
        ak = std::max(ak, (size_t)cap * cand[i] * 4);
    }
    return 5 * 256 + 256 + align_up(conv, 256) + align_up(spmm, 256) + align_up(am, 256) + 2 * align_up(ak, 256);
}

extern "C" insum_status insum_choose_group_size(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* row,
                                                const int32_t* col, const void* val, insum_dtype dt,
                                                const void* B, int64_t ldb, void* C, int64_t ldc,
                                                insum_dtype c_dt, int32_t repeats, int32_t* best_g,
                                                int32_t* candidates, float* candidate_ms,
                                                int32_t* num_candidates, void* workspace,
                                                size_t workspace_bytes, void* stream) {
    if (!best_g || M < 0 || K < 0 || N < 0 || nnz < 0 || repeats <= 0 || !dtype_valid(dt) || !dtype_valid(c_dt))
        return INSUM_ERR_INVALID_ARG;
    int32_t cand[3];
    const int32_t nc = insum_group_size_candidates(nnz, M, cand);
    if (num_candidates) *num_candidates = nc;
    for (int32_t i = 0; i < nc; ++i) {
        if (candidates) candidates[i] = cand[i];
        if (candidate_ms) candidate_ms[i] = -1.f;
    }
    *best_g = insum_default_group_size(nnz, M);
    if (nnz == 0 || M == 0 || N == 0) return INSUM_OK;   // nothing to time: the default stands
    if (!B || !C) return INSUM_ERR_INVALID_ARG;
    if (workspace_bytes < insum_choose_group_size_workspace_bytes(M, N, nnz, dt)) return INSUM_ERR_CAPACITY;

    size_t conv_bytes = insum_coo_to_groupcoo_workspace_bytes(M, nnz), spmm_bytes = 0, am_bytes = 0, ak_bytes = 0;
    for (int32_t i = 0; i < nc; ++i) {
        const int64_t cap = group_capacity(M, nnz, cand[i]);
        spmm_bytes = std::max(spmm_bytes, insum_spmm_groupcoo_workspace_bytes(M, N, cap, cand[i]));
        am_bytes = std::max(am_bytes, (size_t)cap * 4);
        ak_bytes = std::max(ak_bytes, (size_t)cap * cand[i] * 4);
    }
    Carve ws(workspace, workspace_bytes);
    void* conv_ws = ws.take(conv_bytes);
    void* spmm_ws = ws.take(spmm_bytes);
    int32_t* AM = static_cast<int32_t*>(ws.take(am_bytes));
    int32_t* AK = static_cast<int32_t*>(ws.take(ak_bytes));
    void* AV = ws.take(ak_bytes);   // values are at most as wide as the int32 columns
    if (!ws.ok) return INSUM_ERR_CAPACITY;

    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t e0, e1;
    INSUM_HIP_TRY(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return INSUM_ERR_HIP;
    }
    insum_status st = INSUM_OK;
    float best_ms = -1.f;
    for (int32_t i = 0; i < nc && st == INSUM_OK; ++i) {
        const int32_t g = cand[i];
        int32_t g_used = 0;
        int64_t G = 0;
        st = insum_coo_to_groupcoo(M, K, nnz, row, col, val, dt, g, &g_used, &G, AM, AK, AV,
                                   group_capacity(M, nnz, g), conv_ws, conv_bytes, stream);
        if (st != INSUM_OK) break;
        // one untimed launch, then `repeats` launches between two events on the caller's stream
        for (int32_t r = -1; r < repeats && st == INSUM_OK; ++r) {
            if (r == 0 && hipEventRecord(e0, s) != hipSuccess) st = INSUM_ERR_HIP;
            if (st == INSUM_OK)
                st = insum_spmm_groupcoo(M, K, N, G, g, AM, AK, AV, dt, B, ldb, dt, C, ldc, c_dt, 0, spmm_ws,
                                         spmm_bytes, stream);
        }
        if (st != INSUM_OK) break;
        float ms = 0.f;
        if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
            st = INSUM_ERR_HIP;
            break;
        }
        ms /= (float)repeats;
        if (candidate_ms) candidate_ms[i] = ms;
        if (best_ms < 0.f || ms < best_ms) {   // ties keep the smaller group size (the smaller format)
            best_ms = ms;
            *best_g = g;
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return st;
}
