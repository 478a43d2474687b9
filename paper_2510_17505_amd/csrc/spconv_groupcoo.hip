// Point-cloud sparse convolution as an indirect Einsum over a kernel map grouped by offset
// (paper: Section 6.4):
//
//     Out[MAPX[p,q], m] += MAPV[p,q] * sum_c In[MAPY[p,q], c] * Weight[MAPZ[p], c, m]
//
// All slots of a group share one weight matrix, so the work is a sequence of small dense
// products (gathered rows of In) x Weight[z] whose result rows are scattered into Out.  The
// paper expresses this as a batched matrix multiply followed by a lazily broadcast atomic add;
// the mapping to gfx950 below is this library's own:
//
//   * The slot array [G*g] is cut into tiles of 32 consecutive slots; a tile is one
//     v_mfma_f32_32x32x16 row block.  A wavefront owns a contiguous range of tiles.  The map
//     is sorted by offset, so a wavefront sees one offset, rarely two.
//   * Weight-stationary registers: the wavefront keeps Weight[z][:, m-tile] as MFMA B
//     fragments in VGPRs (C x 128 halves = 128 registers for C = 128) and reloads them only
//     when the offset changes.  There is no LDS traffic at all.
//   * A fragments are the gathered rows themselves: lane l loads the 16 bytes
//     In[y(l % 32)][16 ks + 8 (l / 32) ...] for every k-step, which is exactly the operand
//     layout of the instruction.  The next tile's rows are requested before the current
//     tile's MFMAs are issued.
//   * A tile whose slots belong to more than one offset (possible where one offset's groups
//     end and the next begin, and for any g that does not divide 32) is processed once per
//     offset with the other slots masked.
//   * Results are scaled by MAPV in fp32 and added to Out with hardware fp32 atomics:
//     32 consecutive floats of one output row per half wavefront.  A zero MAPV (padding)
//     issues no atomic.
//
// Shapes outside the MFMA conditions and fp32 inputs run spconv_general: one thread per
// (slot, m), fp32 FMAs in channel order.
#include <algorithm>

#include "common.h"

namespace insum {
namespace {

typedef short i16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct ConvParams {
    int64_t X, Y, C, M;
    int64_t slots;  // G * g
    int32_t g;
    const int32_t* MAPZ;
    const int32_t* MAPX;
    const int32_t* MAPY;
    const void* MAPV;
    const void* In;
    int64_t ld_in;
    const void* W;
    float* Out;
    int64_t ld_out;
    int64_t tiles;        // ceil(slots / 32)
    int32_t waves_total;  // wavefronts that share the tiles (per m-tile)
};

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

__device__ inline float half_bits_to_float(uint16_t b, __half) {
    return __half2float(__builtin_bit_cast(__half, b));
}
__device__ inline float half_bits_to_float(uint16_t b, bf16_t) { return __uint_as_float((uint32_t)b << 16); }

// Metadata of one tile as held by a wavefront: lanes l and l + 32 both hold slot l % 32.
struct TileMeta {
    int32_t z;  // offset of the slot, -1 for a slot past the end
    int32_t x, y;
    float v;
};

template <typename T>
__device__ inline TileMeta load_meta(const ConvParams& p, int64_t tile, int l32) {
    TileMeta m;
    const int64_t slot = tile * 32 + l32;
    const bool valid = slot < p.slots;
    const int64_t s = valid ? slot : 0;
    m.z = valid ? p.MAPZ[s / p.g] : -1;
    m.x = p.MAPX[s];
    m.y = p.MAPY[s];
    m.v = valid ? half_bits_to_float(static_cast<const uint16_t*>(p.MAPV)[s], T{}) : 0.f;
    return m;
}

// A fragments of a tile: for k-step ks the lane holds channels 16 ks + 8 (lane / 32) + [0, 8)
// of its slot's input row.  A chunk at or past C is read from the row's last chunk instead:
// its products meet weight fragments that are zero there, and In is finite.
template <int KS>
__device__ inline void gather_rows(const ConvParams& p, int32_t y, int half, i16x8 (&a)[KS]) {
    const uint16_t* row = static_cast<const uint16_t*>(p.In) + (int64_t)y * p.ld_in;
    const int last = (int)p.C - 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const int c0 = min(ks * 16 + half * 8, last);
        a[ks] = __builtin_bit_cast(i16x8, *reinterpret_cast<const u32x4*>(row + c0));
    }
}

// B fragments of Weight[z][:, m0 .. m0 + 32 NT): lane holds, for k-step ks and column block ni,
// the 8 channels 16 ks + 8 (lane / 32) + [0, 8) of column m0 + 32 ni + lane % 32; zero where
// the channel is at or past C or the column at or past M.  Rows are walked with a running
// pointer so that no per-row address has to be kept.
template <int KS, int NT>
__device__ inline void load_weight(const ConvParams& p, int32_t z, int m0, int half, int l32, int ksteps,
                                   i16x8 (&w)[KS][NT]) {
    const uint16_t* wz = static_cast<const uint16_t*>(p.W) + (int64_t)z * p.C * p.M;
    bool col_ok[NT];
    int64_t col[NT];
#pragma unroll
    for (int ni = 0; ni < NT; ++ni) {
        const int64_t m = m0 + ni * 32 + l32;
        col_ok[ni] = m < p.M;
        col[ni] = col_ok[ni] ? m : p.M - 1;
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        if (ks < ksteps) {
            const int c0 = ks * 16 + half * 8;
            const bool chunk_ok = c0 < p.C;  // C % 8 == 0: a chunk is inside or outside as a whole
            const uint16_t* rowp = wz + (int64_t)(chunk_ok ? c0 : 0) * p.M;
            i16x8 frag[NT];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
#pragma unroll
                for (int ni = 0; ni < NT; ++ni) frag[ni][i] = (short)rowp[col[ni]];
                rowp += p.M;
            }
#pragma unroll
            for (int ni = 0; ni < NT; ++ni) {
                const bool ok = chunk_ok && col_ok[ni];
#pragma unroll
                for (int i = 0; i < 8; ++i) w[ks][ni][i] = ok ? frag[ni][i] : (short)0;
            }
        }
    }
}

// grid: x = work-groups of 4 wavefronts over the tiles, y = m-tiles of 32*NT output channels.
// Needs: 16-bit T, C % 8 == 0, 8 <= C <= 16 KS, ld_in % 8 == 0, In 16-byte aligned.
template <typename T, int KS, int NT>
__global__ __launch_bounds__(256, 1) void spconv_mfma(ConvParams p) {
    const int lane = threadIdx.x % 64;
    const int half = lane / 32, l32 = lane % 32;
    const int64_t wave = (int64_t)blockIdx.x * 4 + threadIdx.x / 64;
    const int m0 = blockIdx.y * 32 * NT;
    const int64_t t0 = p.tiles * wave / p.waves_total;
    const int64_t t1 = p.tiles * (wave + 1) / p.waves_total;
    if (t0 >= t1) return;
    const int ksteps = (int)((p.C + 15) / 16);
    const bool m_full = m0 + 32 * NT <= p.M;  // every column block of this m-tile is inside M
    float* const out_col = p.Out + m0 + l32;

    i16x8 w[KS][NT];
    int32_t z_loaded = -1;

    TileMeta cur = load_meta<T>(p, t0, l32);
    i16x8 a[KS];
    gather_rows<KS>(p, cur.y, half, a);

    for (int64_t t = t0; t < t1; ++t) {
        // request the next tile's rows before this tile's arithmetic
        TileMeta nxt = cur;
        i16x8 a_next[KS];
        if (t + 1 < t1) {
            nxt = load_meta<T>(p, t + 1, l32);
            gather_rows<KS>(p, nxt.y, half, a_next);
        } else {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) a_next[ks] = a[ks];
        }

        uint32_t remaining = (uint32_t)__ballot(cur.z >= 0);  // low half: one bit per slot
        while (remaining) {
            const int first = __builtin_ctz(remaining);
            const int32_t zc = __builtin_amdgcn_readlane(cur.z, first);
            const bool mine = cur.z == zc;
            remaining &= ~(uint32_t)__ballot(mine);
            if (zc != z_loaded) {
                load_weight<KS, NT>(p, zc, m0, half, l32, ksteps, w);
                z_loaded = zc;
            }
            f32x16 acc[NT];
#pragma unroll
            for (int ni = 0; ni < NT; ++ni)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[ni][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (ks < ksteps) {
#pragma unroll
                    for (int ni = 0; ni < NT; ++ni) acc[ni] = mfma32<T>(a[ks], w[ks][ni], acc[ni]);
                }
            }
            // accumulator register r of this lane is slot 8 (r / 4) + 4 (lane / 32) + r % 4,
            // output channel m0 + 32 ni + lane % 32
            const float v_masked = mine ? cur.v : 0.f;
            const bool dense = m_full && (uint32_t)__ballot(v_masked != 0.f) == 0xffffffffu;
            if (dense) {  // every slot of the tile adds to every column: no per-lane guards
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int srow = 8 * (r / 4) + 4 * half + (r % 4);
                    const float vr = __shfl(v_masked, srow);
                    float* out = out_col + (int64_t)__shfl(cur.x, srow) * p.ld_out;
#pragma unroll
                    for (int ni = 0; ni < NT; ++ni) unsafeAtomicAdd(out + ni * 32, vr * acc[ni][r]);
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int srow = 8 * (r / 4) + 4 * half + (r % 4);
                    const float vr = __shfl(v_masked, srow);
                    float* out = out_col + (int64_t)__shfl(cur.x, srow) * p.ld_out;
                    if (vr != 0.f) {
#pragma unroll
                        for (int ni = 0; ni < NT; ++ni)
                            if (m0 + ni * 32 + l32 < p.M) unsafeAtomicAdd(out + ni * 32, vr * acc[ni][r]);
                    }
                }
            }
        }
        cur = nxt;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) a[ks] = a_next[ks];
    }
}

// One thread per (slot, output channel): any dtype, any shape.
// grid: x = ceil(slots / kSlotsPerBlock), y = ceil(M / 256); block = 256 threads over m.
constexpr int kSlotsPerBlock = 8;

template <typename T>
__global__ __launch_bounds__(256) void spconv_general(ConvParams p) {
    const int64_t m = (int64_t)blockIdx.y * 256 + threadIdx.x;
    if (m >= p.M) return;
    const T* In = static_cast<const T*>(p.In);
    const T* W = static_cast<const T*>(p.W);
    const T* V = static_cast<const T*>(p.MAPV);
    const int64_t s0 = (int64_t)blockIdx.x * kSlotsPerBlock;
    for (int64_t s = s0; s < s0 + kSlotsPerBlock && s < p.slots; ++s) {
        const float v = to_float(V[s]);
        if (v == 0.f) continue;
        const T* in = In + (int64_t)p.MAPY[s] * p.ld_in;
        const T* w = W + (int64_t)p.MAPZ[s / p.g] * p.C * p.M + m;
        float acc = 0.f;
        for (int64_t c = 0; c < p.C; ++c) acc = fmaf(to_float(in[c]), to_float(w[c * p.M]), acc);
        unsafeAtomicAdd(p.Out + (int64_t)p.MAPX[s] * p.ld_out + m, v * acc);
    }
}

__global__ void fill_zero_rows(float* out, int64_t rows, int64_t cols, int64_t ld) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= rows * cols) return;
    out[(i / cols) * ld + (i % cols)] = 0.f;
}

template <typename T, int KS, int NT>
void launch_mfma(ConvParams p, hipStream_t s) {
    const int64_t m_tiles = ceil_div(p.M, 32 * NT);
    // one work-group of four wavefronts per compute unit (the register budget allows one
    // wavefront per SIMD), fewer when there are fewer tiles
    const int64_t groups = std::min<int64_t>(ceil_div(p.tiles, 4), 256 * 2);
    p.waves_total = (int32_t)(groups * 4);
    hipLaunchKernelGGL((spconv_mfma<T, KS, NT>), dim3((unsigned)groups, (unsigned)m_tiles), dim3(256), 0, s, p);
}

template <typename T>
void launch_typed(const ConvParams& p, bool mfma_ok, hipStream_t s) {
    if constexpr (sizeof(T) == 2) {
        if (mfma_ok) {
            if (p.C <= 32) return launch_mfma<T, 2, 4>(p, s);
            if (p.C <= 64) return launch_mfma<T, 4, 4>(p, s);
            if (p.C <= 128) return launch_mfma<T, 8, 4>(p, s);
            return launch_mfma<T, 16, 2>(p, s);
        }
    }
    hipLaunchKernelGGL(spconv_general<T>, dim3((unsigned)ceil_div(p.slots, kSlotsPerBlock),
                                               (unsigned)ceil_div(p.M, 256)),
                       dim3(256), 0, s, p);
}

}  // namespace
}  // namespace insum

using namespace insum;

extern "C" insum_status insum_spconv_groupcoo(int64_t X, int64_t Y, int64_t Z, int64_t C, int64_t M,
                                              int64_t G, int32_t g, const int32_t* MAPZ,
                                              const int32_t* MAPX, const int32_t* MAPY, const void* MAPV,
                                              const void* In, int64_t ld_in, const void* W, insum_dtype dt,
                                              float* Out, int64_t ld_out, int accumulate, void* stream) {
    if (X < 0 || Y < 0 || Z < 0 || C < 0 || M < 0 || G < 0 || g <= 0) return INSUM_ERR_INVALID_ARG;
    if (X >= (1LL << 31) || Y >= (1LL << 31) || Z >= (1LL << 31) || C >= (1LL << 31) || M >= (1LL << 31))
        return INSUM_ERR_INVALID_ARG;
    if (!dtype_valid(dt) || ld_in < C || ld_out < M) return INSUM_ERR_INVALID_ARG;
    if (G * (int64_t)g >= (1LL << 40)) return INSUM_ERR_INVALID_ARG;
    if (X > 0 && M > 0 && !Out) return INSUM_ERR_INVALID_ARG;
    if (G > 0 && (!MAPZ || !MAPX || !MAPY || !MAPV)) return INSUM_ERR_INVALID_ARG;
    if (G > 0 && C > 0 && M > 0 && (!In || !W)) return INSUM_ERR_INVALID_ARG;
    if (G > 0 && (X == 0 || Y == 0 || Z == 0)) return INSUM_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (X == 0 || M == 0) return INSUM_OK;
    if (!accumulate) {
        const int64_t n = X * M;
        hipLaunchKernelGGL(fill_zero_rows, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s, Out, X, M, ld_out);
    }
    if (G > 0 && C > 0) {
        ConvParams p;
        p.X = X, p.Y = Y, p.C = C, p.M = M;
        p.slots = G * (int64_t)g;
        p.g = g;
        p.MAPZ = MAPZ, p.MAPX = MAPX, p.MAPY = MAPY, p.MAPV = MAPV;
        p.In = In, p.ld_in = ld_in, p.W = W, p.Out = Out, p.ld_out = ld_out;
        p.tiles = ceil_div(p.slots, 32);
        p.waves_total = 0;
        const bool mfma_ok = dt != INSUM_F32 && C % 8 == 0 && C >= 8 && C <= 256 && ld_in % 8 == 0 &&
                             reinterpret_cast<uintptr_t>(In) % 16 == 0 &&
                             ceil_div(M, 64) < 65536 && ceil_div(p.slots, kSlotsPerBlock) < (1LL << 31);
        if (ceil_div(M, 256) >= 65536 || ceil_div(p.slots, kSlotsPerBlock) >= (1LL << 31))
            return INSUM_ERR_UNSUPPORTED;
        if (dt == INSUM_F32) launch_typed<float>(p, false, s);
        else if (dt == INSUM_F16) launch_typed<__half>(p, mfma_ok, s);
        else launch_typed<bf16_t>(p, mfma_ok, s);
    }
    INSUM_HIP_TRY(hipGetLastError());
    return INSUM_OK;
}
