// SpMM over BlockGroupCOO for gfx950:
//     C[AM[p]*bM + bm, n] (+)= sum_{q,bk} AV[p,q,bm,bk] * B[AK[p,q]*bK + bk, n]
// (paper: Section 4.1, BlockGroupCOO Einsum; the fused gather - dot - scatter structure of
// the generated kernel in Section 5.2: the whole reduction of an output tile is kept on
// chip and the tile is written once).
//
// MFMA kernel
//   * One workgroup (4 wavefronts) owns one block row x 256 output columns; each wavefront
//     owns 64 of those columns and keeps its bM x 64 fp32 accumulator in registers for the
//     whole block row, so C is written exactly once and never needs atomics.
//   * The groups of a block row are consecutive in AM (it is non-decreasing); the workgroup
//     finds them by binary search.  A block row without groups just writes zeros.
//   * For every stored block (padding blocks repeat the previous block column and are
//     skipped) and every k-chunk of KC <= 64 rows: the gathered B tile (KC x 256) is
//     fetched with 16-byte loads, 512 contiguous bytes per row, and staged in LDS (double
//     buffered, one barrier per step, the next tile's loads in flight during the MFMAs).
//   * B is row-major (n fastest) but the MFMA B operand wants 8 consecutive k per lane:
//     the transposing LDS read ds_read_b64_tr_b16 delivers exactly that (16 lanes read a
//     4(k) x 16(n) patch and receive 4 k-values of one column each).  LDS rows are padded
//     by 64 bytes so the four rows of a patch fall into different banks.
//   * AV blocks are k-contiguous, which is the MFMA A operand layout: each lane loads its
//     8 k-values (16 bytes) straight from global memory, no staging.
//   * v_mfma_f32_32x32x16_{bf16,f16}: A lane l -> row l%32, k = 8*(l/32)..+7;
//     B lane l -> column l%32, same k; D register r -> row 8*(r/4) + 4*(l/32) + r%4,
//     column l%32.
//
// General kernel: any block shape and dtype, one thread per output column, plain fp32 FMAs.
#include <algorithm>

#include "common.h"

namespace insum {
namespace {

struct BlockParams {
    int64_t M, N, G;
    int32_t g, bM, bK;
    const int32_t* AM;
    const int32_t* AK;
    const void* AV;
    const void* B;
    int64_t ldb;
    void* C;
    int64_t ldc;
    int32_t accumulate;
};

typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef short i16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ inline int64_t lower_bound_i32(const int32_t* a, int64_t n, int32_t v) {
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (a[mid] < v) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

template <typename T>
__device__ inline f32x16 mfma32(i16x8 a, i16x8 b, f32x16 c);
template <>
__device__ inline f32x16 mfma32<bf16_t>(i16x8 a, i16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
template <>
__device__ inline f32x16 mfma32<__half>(i16x8 a, i16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                  __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

constexpr int kTileN = 256;              // output columns per workgroup
constexpr int kWaveN = 64;               // output columns per wavefront
constexpr int kLdsStride = kTileN + 32;  // elements per LDS row (512 B of data + 64 B pad)

// Walks the stored blocks of one block row, k-chunk by k-chunk, skipping padding blocks.
struct StepIter {
    const int32_t* AK;
    int64_t slot, slot_end;  // flat slot index p*g+q
    int32_t g, kc, kchunks;
    int32_t col;             // block column of the current slot
    __device__ bool valid() const { return slot < slot_end; }
    __device__ void settle() {  // move forward to a slot that is not padding
        while (slot < slot_end) {
            col = AK[slot];
            if ((slot % g) == 0 || AK[slot - 1] != col) break;
            ++slot;
        }
    }
    __device__ void next() {
        if (++kc == kchunks) {
            kc = 0;
            ++slot;
            settle();
        }
    }
};

template <typename T, typename TC, int BM, int KC>
__global__ __launch_bounds__(256) void spmm_block_mfma(BlockParams p) {
    constexpr int MI = BM / 32;      // 32-row MFMA tiles per block
    constexpr int KS = KC / 16;      // MFMA k-steps per chunk
    constexpr int NI = kWaveN / 32;  // 32-column MFMA tiles per wavefront
    constexpr int LOADS = KC / 8;    // 16-byte B loads per thread and chunk
    __shared__ __attribute__((aligned(16))) uint16_t lds[2][KC][kLdsStride];

    const int tid = threadIdx.x;
    const int lane = tid % 64;
    const int wave = tid / 64;
    const int64_t brow = blockIdx.x;
    const int64_t ntile0 = (int64_t)blockIdx.y * kTileN;

    const uint16_t* __restrict__ AV = static_cast<const uint16_t*>(p.AV);
    const uint16_t* __restrict__ B = static_cast<const uint16_t*>(p.B);
    TC* C = static_cast<TC*>(p.C);

    const int64_t p0 = lower_bound_i32(p.AM, p.G, (int32_t)brow);
    const int64_t p1 = lower_bound_i32(p.AM, p.G, (int32_t)brow + 1);

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    StepIter it;
    it.AK = p.AK;
    it.slot = p0 * p.g;
    it.slot_end = p1 * p.g;
    it.g = p.g;
    it.kc = 0;
    it.kchunks = p.bK / KC;
    it.col = 0;
    it.settle();

    // B tile: thread -> 16-byte column chunk (tid % 32) of rows tid/32 + 8*i
    const int bcol = (tid % 32) * 8;
    const int brow0 = tid / 32;
    const bool bcol_ok = ntile0 + bcol < p.N;
    u32x4 breg[LOADS];
    auto load_b = [&](const StepIter& s) {
        const int64_t krow = (int64_t)s.col * p.bK + (int64_t)s.kc * KC + brow0;
        const uint16_t* src = B + krow * p.ldb + ntile0 + bcol;
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            if (bcol_ok) breg[i] = *reinterpret_cast<const u32x4*>(src + (int64_t)(8 * i) * p.ldb);
            else breg[i] = u32x4{0, 0, 0, 0};
        }
    };
    auto store_b = [&](int buf) {
#pragma unroll
        for (int i = 0; i < LOADS; ++i)
            *reinterpret_cast<u32x4*>(&lds[buf][brow0 + 8 * i][bcol]) = breg[i];
    };
    // A fragments: lane -> row lane%32 of each 32-row tile, 8 k-values at 8*(lane/32)
    auto load_a = [&](const StepIter& s, i16x8 (&a)[MI][KS]) {
        const uint16_t* blk = AV + s.slot * (int64_t)p.bM * p.bK + (int64_t)s.kc * KC;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                a[mi][ks] = *reinterpret_cast<const i16x8*>(
                    blk + (int64_t)(32 * mi + lane % 32) * p.bK + 16 * ks + 8 * (lane / 32));
    };
    // B fragment patch addressing for the transposing LDS read
    const int tr_row = 8 * (lane / 32) + (lane % 16) / 4;                       // + 16*ks + 4*r
    const int tr_col = kWaveN * wave + 16 * ((lane / 16) % 2) + 4 * (lane % 4);  // + 32*ni
    auto compute = [&](int buf, const i16x8 (&a)[MI][KS]) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                typedef i16x4 __attribute__((address_space(3))) * lds_ptr;
                const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (lds_ptr)(&lds[buf][16 * ks + tr_row][tr_col + 32 * ni]));
                const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (lds_ptr)(&lds[buf][16 * ks + tr_row + 4][tr_col + 32 * ni]));
                const i16x8 b = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) acc[mi][ni] = mfma32<T>(a[mi][ks], b, acc[mi][ni]);
            }
        }
    };

    if (it.valid()) {
        i16x8 a0[MI][KS], a1[MI][KS];
        load_b(it);
        load_a(it, a0);
        int buf = 0;
        while (true) {
            store_b(buf);
            __syncthreads();
            it.next();
            if (it.valid()) {
                load_b(it);
                load_a(it, a1);
            }
            compute(buf, a0);
            buf ^= 1;
            if (!it.valid()) break;

            store_b(buf);
            __syncthreads();
            it.next();
            if (it.valid()) {
                load_b(it);
                load_a(it, a0);
            }
            compute(buf, a1);
            buf ^= 1;
            if (!it.valid()) break;
        }
    }

    // epilogue: one store per output element (block rows without groups store zeros)
    const bool accumulate = p.accumulate != 0;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int64_t col = ntile0 + kWaveN * wave + 32 * ni + lane % 32;
            if (col < p.N) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t row = brow * BM + 32 * mi + 8 * (r / 4) + 4 * (lane / 32) + r % 4;
                    TC* dst = C + row * p.ldc + col;
                    float v = acc[mi][ni][r];
                    if (accumulate) v += to_float(*dst);
                    *dst = from_float<TC>(v);
                }
            }
        }
}

// ---- general kernel ------------------------------------------------------------------------
template <typename T, typename TC>
__global__ __launch_bounds__(256) void spmm_block_general(BlockParams p) {
    const int64_t brow = blockIdx.x;
    const int64_t n = (int64_t)blockIdx.y * 256 + threadIdx.x;
    if (n >= p.N) return;
    const T* __restrict__ AV = static_cast<const T*>(p.AV);
    const T* __restrict__ B = static_cast<const T*>(p.B);
    TC* C = static_cast<TC*>(p.C);
    const int64_t p0 = lower_bound_i32(p.AM, p.G, (int32_t)brow);
    const int64_t p1 = lower_bound_i32(p.AM, p.G, (int32_t)brow + 1);
    for (int32_t bm = 0; bm < p.bM; ++bm) {
        float acc = 0.f;
        for (int64_t slot = p0 * p.g; slot < p1 * p.g; ++slot) {
            const int32_t col = p.AK[slot];
            if ((slot % p.g) != 0 && p.AK[slot - 1] == col) continue;  // padding block
            const T* arow = AV + (slot * p.bM + bm) * (int64_t)p.bK;
            const T* bcolp = B + (int64_t)col * p.bK * p.ldb + n;
            for (int32_t bk = 0; bk < p.bK; ++bk)
                acc = fmaf(to_float(arow[bk]), to_float(bcolp[(int64_t)bk * p.ldb]), acc);
        }
        TC* dst = C + (brow * p.bM + bm) * p.ldc + n;
        if (p.accumulate) acc += to_float(*dst);
        *dst = from_float<TC>(acc);
    }
}

template <typename T, typename TC, int BM>
void launch_mfma_kc(const BlockParams& p, dim3 grid, hipStream_t s) {
    if (p.bK % 64 == 0) hipLaunchKernelGGL((spmm_block_mfma<T, TC, BM, 64>), grid, dim3(256), 0, s, p);
    else if (p.bK % 32 == 0) hipLaunchKernelGGL((spmm_block_mfma<T, TC, BM, 32>), grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((spmm_block_mfma<T, TC, BM, 16>), grid, dim3(256), 0, s, p);
}

template <typename T, typename TC>
void launch_typed(const BlockParams& p, bool mfma_ok, hipStream_t s) {
    const dim3 grid((unsigned)(p.M / p.bM), (unsigned)ceil_div(p.N, kTileN));
    if constexpr (sizeof(T) == 2) {
        if (mfma_ok && p.bM == 32) return launch_mfma_kc<T, TC, 32>(p, grid, s);
        if (mfma_ok && p.bM == 64) return launch_mfma_kc<T, TC, 64>(p, grid, s);
    }
    hipLaunchKernelGGL((spmm_block_general<T, TC>), grid, dim3(256), 0, s, p);
}

}  // namespace
}  // namespace insum

using namespace insum;

extern "C" size_t insum_spmm_blockgroupcoo_workspace_bytes(int64_t, int64_t, int64_t, int32_t,
                                                           int32_t, int32_t) {
    return 0;  // every output tile is owned by one workgroup: no scratch is needed
}

extern "C" insum_status insum_spmm_blockgroupcoo(int64_t M, int64_t K, int64_t N, int64_t G,
                                                 int32_t g, int32_t bM, int32_t bK,
                                                 const int32_t* AM, const int32_t* AK,
                                                 const void* AV, insum_dtype a_dt, const void* B,
                                                 int64_t ldb, insum_dtype b_dt, void* C,
                                                 int64_t ldc, insum_dtype c_dt, int accumulate,
                                                 void* workspace, size_t workspace_bytes,
                                                 void* stream) {
    (void)workspace;
    (void)workspace_bytes;
    if (M < 0 || K < 0 || N < 0 || G < 0 || g <= 0 || bM <= 0 || bK <= 0) return INSUM_ERR_INVALID_ARG;
    if (M >= (1LL << 31) || K >= (1LL << 31) || N >= (1LL << 31)) return INSUM_ERR_INVALID_ARG;
    if (!dtype_valid(a_dt) || !dtype_valid(b_dt) || !dtype_valid(c_dt)) return INSUM_ERR_INVALID_ARG;
    if (a_dt != b_dt || (c_dt != b_dt && c_dt != INSUM_F32)) return INSUM_ERR_UNSUPPORTED;
    if (M % bM || K % bK) return INSUM_ERR_UNSUPPORTED;
    if (ldb < N || ldc < N) return INSUM_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return INSUM_OK;
    if (!C) return INSUM_ERR_INVALID_ARG;
    if (G > 0 && (!AM || !AK || !AV || !B || K == 0)) return INSUM_ERR_INVALID_ARG;
    if (M / bM > 0x7fffffffLL / 2) return INSUM_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);

    BlockParams p;
    p.M = M; p.N = N; p.G = G; p.g = g; p.bM = bM; p.bK = bK;
    p.AM = AM; p.AK = AK; p.AV = AV; p.B = B; p.ldb = ldb; p.C = C; p.ldc = ldc;
    p.accumulate = accumulate ? 1 : 0;

    const bool mfma_ok = bK % 16 == 0 && bK <= 128 && N % 8 == 0 && ldb % 8 == 0 &&
                         (reinterpret_cast<uintptr_t>(B) % 16) == 0 &&
                         (reinterpret_cast<uintptr_t>(AV) % 16) == 0;
    if (b_dt == INSUM_F32) launch_typed<float, float>(p, false, s);
    else if (b_dt == INSUM_F16 && c_dt == INSUM_F16) launch_typed<__half, __half>(p, mfma_ok, s);
    else if (b_dt == INSUM_F16) launch_typed<__half, float>(p, mfma_ok, s);
    else if (c_dt == INSUM_BF16) launch_typed<bf16_t, bf16_t>(p, mfma_ok, s);
    else launch_typed<bf16_t, float>(p, mfma_ok, s);
    INSUM_HIP_TRY(hipGetLastError());
    return INSUM_OK;
}
