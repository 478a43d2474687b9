// Product with the transposed matrix over the stored GroupCOO format, for gfx950:
//     D[AK[p,q], n] (+)= AV[p,q] * E[AM[p], n]            (D = A^T * E)
// the Section 4.1 Einsum with the dense operands exchanged - the derivative of the SpMM with
// respect to its dense operand (Section 5.1 gives autodiff as a reason for the Einsum form).
//
// The format is grouped along the rows of A, which here are the rows of the *input* E: a group's
// row of E is loaded once and serves its g slots (the format's advantage on this side), while
// the contributions to one row of D come from slots scattered over the whole format.  Without a
// second, column-grouped copy of A they can only be combined in memory, so they are added with
// the hardware fp32 atomics of the L2 (no compare-and-swap loop).  Consequences, all stated in
// the header: sums are formed in fp32 in an order that varies from run to run; a 16-bit D is
// accumulated in an fp32 workspace and rounded once by a final pass; D (or the workspace) is
// cleared first when the call does not accumulate.
//
// Work split: the group list is cut into equal runs, one per wavefront.  Slots with value zero
// (padding) are skipped.
#include <algorithm>

#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

#include "common.h"

namespace insum {
namespace {

struct TransposedParams {
    int64_t M, K, N, G;
    int32_t g;
    const int32_t* AM;
    const int32_t* AK;
    const void* AV;
    const void* E;
    int64_t lde;
    float* acc;       // fp32 sums: D itself (fp32 D) or the workspace
    int64_t ld_acc;
    int64_t runs, groups_per_run;
    int32_t col_tiles;
};

// A wavefront owns a run of groups and walks the columns in slabs of 64 * CPL: lane l holds
// columns l, l + 64, ... of the slab, so that one atomic instruction of the wavefront covers 64
// consecutive floats (two whole 128-byte lines; 16-byte pieces per lane would make every
// instruction touch every line of the row, and the L2 works line by line).
template <typename T, int CPL>
__global__ __launch_bounds__(256) void spmm_transposed_scatter(TransposedParams p) {
    const int lane = threadIdx.x % 64;
    const int64_t run = ((int64_t)(blockIdx.x / p.col_tiles) * 256 + threadIdx.x) / 64;
    if (run >= p.runs) return;
    const int64_t n0 = (int64_t)(blockIdx.x % p.col_tiles) * (64 * CPL) + lane;
    const T* __restrict__ E = static_cast<const T*>(p.E);
    const T* __restrict__ AV = static_cast<const T*>(p.AV);
    const int64_t gs = run * p.groups_per_run;
    const int64_t ge = gs + p.groups_per_run < p.G ? gs + p.groups_per_run : p.G;
    for (int64_t grp = gs; grp < ge; ++grp) {
        float e[CPL];
        const T* erow = E + (int64_t)p.AM[grp] * p.lde;   // one row of E per group
#pragma unroll
        for (int i = 0; i < CPL; ++i) e[i] = n0 + 64 * i < p.N ? to_float(erow[n0 + 64 * i]) : 0.f;
        for (int32_t q = 0; q < p.g; ++q) {
            const float a = to_float(AV[grp * p.g + q]);
            if (a == 0.f) continue;   // padding (and explicit zeros) add nothing; uniform in the wavefront
            float* dst = p.acc + (int64_t)p.AK[grp * p.g + q] * p.ld_acc + n0;
#pragma unroll
            for (int i = 0; i < CPL; ++i)
                if (n0 + 64 * i < p.N) unsafeAtomicAdd(dst + 64 * i, a * e[i]);
        }
    }
}

template <typename T>
__global__ __launch_bounds__(256) void fill_zero_rows(T* dst, int64_t ld, int64_t rows, int64_t cols) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= rows * cols) return;
    dst[(i / cols) * ld + (i % cols)] = from_float<T>(0.f);
}

// D = round(acc) or round(D + acc), for a 16-bit D
template <typename T>
__global__ __launch_bounds__(256) void round_sums(const float* __restrict__ acc, int64_t ld_acc, T* D, int64_t ldd,
                                                  int64_t rows, int64_t cols, int accumulate) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= rows * cols) return;
    const int64_t r = i / cols, c = i % cols;
    float v = acc[r * ld_acc + c];
    if (accumulate) v += to_float(D[r * ldd + c]);
    D[r * ldd + c] = from_float<T>(v);
}

int64_t padded_cols(int64_t N) { return (N + 7) / 8 * 8; }

template <typename T, int CPL>
void launch_scatter(TransposedParams& p, hipStream_t s) {
    p.col_tiles = (int32_t)ceil_div(p.N, 64 * CPL);
    // about two runs per wavefront slot of the chip
    const int64_t target_runs = std::max<int64_t>(1, 2 * 256LL * 32 / p.col_tiles);
    p.groups_per_run = std::max<int64_t>(1, ceil_div(p.G, target_runs));
    p.runs = ceil_div(p.G, p.groups_per_run);
    const int64_t blocks = ceil_div(p.runs, 4) * p.col_tiles;
    hipLaunchKernelGGL((spmm_transposed_scatter<T, CPL>), dim3((unsigned)blocks), dim3(256), 0, s, p);
}

template <typename T>
void launch_typed(TransposedParams& p, hipStream_t s) {
    if (p.N <= 64) return launch_scatter<T, 1>(p, s);
    if (p.N <= 128) return launch_scatter<T, 2>(p, s);
    return launch_scatter<T, 4>(p, s);
}

}  // namespace
}  // namespace insum

using namespace insum;

extern "C" size_t insum_spmm_groupcoo_transposed_workspace_bytes(int64_t K, int64_t N, insum_dtype d_dt) {
    if (K <= 0 || N <= 0 || d_dt == INSUM_F32) return 0;
    return (size_t)K * (size_t)padded_cols(N) * sizeof(float) + 256;
}

extern "C" insum_status insum_spmm_groupcoo_transposed(int64_t M, int64_t K, int64_t N, int64_t G, int32_t g,
                                                       const int32_t* AM, const int32_t* AK, const void* AV,
                                                       insum_dtype a_dt, const void* E, int64_t lde,
                                                       insum_dtype e_dt, void* D, int64_t ldd, insum_dtype d_dt,
                                                       int accumulate, void* workspace, size_t workspace_bytes,
                                                       void* stream) {
    if (M < 0 || K < 0 || N < 0 || G < 0 || g <= 0) return INSUM_ERR_INVALID_ARG;
    if (M >= (1LL << 31) || K >= (1LL << 31) || N >= (1LL << 31)) return INSUM_ERR_INVALID_ARG;
    if (!dtype_valid(a_dt) || !dtype_valid(e_dt) || !dtype_valid(d_dt)) return INSUM_ERR_INVALID_ARG;
    if (a_dt != e_dt || (d_dt != e_dt && d_dt != INSUM_F32)) return INSUM_ERR_UNSUPPORTED;
    if (lde < N || ldd < N) return INSUM_ERR_INVALID_ARG;
    if (K == 0 || N == 0) return INSUM_OK;
    if (!D) return INSUM_ERR_INVALID_ARG;
    if (G > 0 && (!AM || !AK || !AV || !E || M == 0)) return INSUM_ERR_INVALID_ARG;
    if (ceil_div(K * padded_cols(N), 256) >= (1LL << 31)) return INSUM_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned elem_blocks = (unsigned)ceil_div(K * N, 256);

    TransposedParams p{};
    p.M = M; p.K = K; p.N = N; p.G = G; p.g = g;
    p.AM = AM; p.AK = AK; p.AV = AV; p.E = E; p.lde = lde;
    const bool direct = d_dt == INSUM_F32;   // atomics go straight into D
    if (direct) {
        p.acc = static_cast<float*>(D);
        p.ld_acc = ldd;
        if (!accumulate)
            hipLaunchKernelGGL(fill_zero_rows<float>, dim3(elem_blocks), dim3(256), 0, s, p.acc, ldd, K, N);
    } else {
        const uintptr_t base = reinterpret_cast<uintptr_t>(workspace);
        const uintptr_t ws = (base + 255) / 256 * 256;
        p.ld_acc = padded_cols(N);
        if (!workspace || ws + (size_t)K * p.ld_acc * sizeof(float) > base + workspace_bytes) return INSUM_ERR_CAPACITY;
        p.acc = reinterpret_cast<float*>(ws);
        hipLaunchKernelGGL(fill_zero_rows<float>, dim3(elem_blocks), dim3(256), 0, s, p.acc, p.ld_acc, K, N);
    }
    if (G > 0) {
        if (e_dt == INSUM_F32) launch_typed<float>(p, s);
        else if (e_dt == INSUM_F16) launch_typed<__half>(p, s);
        else launch_typed<bf16_t>(p, s);
    }
    if (!direct) {
        if (d_dt == INSUM_F16)
            hipLaunchKernelGGL(round_sums<__half>, dim3(elem_blocks), dim3(256), 0, s, (const float*)p.acc, p.ld_acc,
                               static_cast<__half*>(D), ldd, K, N, accumulate ? 1 : 0);
        else
            hipLaunchKernelGGL(round_sums<bf16_t>, dim3(elem_blocks), dim3(256), 0, s, (const float*)p.acc, p.ld_acc,
                               static_cast<bf16_t*>(D), ldd, K, N, accumulate ? 1 : 0);
    }
    INSUM_HIP_TRY(hipGetLastError());
    return INSUM_OK;
}
