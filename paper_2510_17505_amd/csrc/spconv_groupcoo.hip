// Point-cloud sparse convolution as an indirect Einsum over a kernel map grouped by offset
// (paper: Section 6.4):
//
//     Out[MAPX[p,q], m] += MAPV[p,q] * sum_c In[MAPY[p,q], c] * Weight[MAPZ[p], c, m]
//
// All slots of a group share one weight matrix, so the work is a sequence of small dense
// products (gathered rows of In) x Weight[z] whose result rows are added into Out.  The paper
// expresses this as a batched matrix multiply followed by a lazily broadcast atomic add.  This
// file holds two mappings of it to gfx950, both this library's own, and a general fallback:
//
//   spconv_os       output-stationary: the grouped map is walked by output point and the sums
//                   stay in registers (described further down, above OsParams).  Used when
//                   the map holds at least X*Z/16 slots.
//   spconv_mfma     slot-major with an atomic scatter, the paper's shape:
//     * The slot array [G*g] is cut into tiles of 32 consecutive slots; a tile is one
//       v_mfma_f32_32x32x16 row block.  A wavefront owns a contiguous range of tiles.  The map
//       is sorted by offset, so a wavefront sees one offset, rarely two.
//     * Weight-stationary registers: the wavefront keeps Weight[z][:, m-tile] as MFMA B
//       fragments in VGPRs (C x 128 halves = 128 registers for C = 128) and reloads them only
//       when the offset changes.  There is no LDS traffic at all.
//     * A fragments are the gathered rows themselves: lane l loads the 16 bytes
//       In[y(l % 32)][16 ks + 8 (l / 32) ...] for every k-step, which is exactly the operand
//       layout of the instruction.  The next tile's rows are requested before the current
//       tile's MFMAs are issued.
//     * A tile whose slots belong to more than one offset (possible where one offset's groups
//       end and the next begin, and for any g that does not divide 32) is processed once per
//       offset with the other slots masked.
//     * Results are scaled by MAPV in fp32 and added to Out with hardware fp32 atomics:
//       32 consecutive floats of one output row per half wavefront.  A zero MAPV (padding)
//       issues no atomic.
//   spconv_general  one thread per (slot, m), fp32 FMAs in channel order, atomics: fp32 inputs
//                   and shapes outside the MFMA conditions.
#include <algorithm>
#include <type_traits>

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

// ---------------------------------------------------------------------------------------------
// Output-stationary schedule.
//
// fp32 atomics complete at a fixed rate in the L2 (about two floats per clock and channel), which
// bounds the scatter kernel above at roughly S*M / 6e11 seconds.  When the map is dense enough
// (a few entries per 32 output points and offset) it is cheaper to walk the same grouped map
// by output point: a work-group owns 32 consecutive output points per wavefront (128 or 256) and
// 64 or 128 output channels, visits every offset once, and keeps the sums in registers until
// they are stored once.  Three small kernels prepare this per call, all in the caller's workspace:
//   * table_fill / table_build invert the map into tabY[z][x] (input point or -1) and
//     tabV[z][x]: one thread per slot claims its cell with a compare-and-swap.  A slot that
//     finds the cell taken (the same (x, z) twice) goes to an overflow list.
//   * weight_transpose writes Wt[z][m][c], zero-padded to whole tiles, so that the MFMA B
//     fragment (8 consecutive channels of one output channel) is one 16-byte read.
// spconv_os stages Wt[z] for its output channels in LDS (double-buffered, rows swizzled so
// that the 16-byte fragment reads of 16 neighbouring output channels hit all 64 banks once),
// gathers the rows In[tabY[z][x]] straight into A fragments (absent points contribute zero
// rows) and runs the k-steps, either straight into the running sums or into a fresh
// accumulator that is scaled by tabV first (the two variants below).  Table entries are read
// two offsets ahead, rows and weights one offset ahead.
// spconv_overflow then adds the overflow list's contributions with atomics.
// ---------------------------------------------------------------------------------------------
struct OsParams {
    int64_t X, Z, C, M;
    int64_t Xp;           // X rounded up to a multiple of 512 (table row length)
    int32_t* tabY;        // [Z][Xp]
    uint16_t* tabV;       // [Z][Xp]
    uint16_t* Wt;         // [Z][Mp][Cp]
    int64_t Mp;           // M rounded up to a multiple of 128
    int32_t Cp;           // 16 * KS
    int32_t* ovf_count;   // one counter
    int32_t* nonunit;     // set when some nonzero map value differs from 1
    int32_t* ovf;         // [slots] slot ids
    const void* In;
    int64_t ld_in;
    float* Out;
    int64_t ld_out;
    int32_t accumulate;
    int32_t m_tiles, x_blocks;
};

__global__ void table_fill(OsParams o) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < o.Z * o.Xp) o.tabY[i] = -1;
    if (i == 0) *o.ovf_count = 0, *o.nonunit = 0;
}

// one_bits: the bit pattern of 1.0 in the map's value type
__global__ void table_build(ConvParams p, OsParams o, uint16_t one_bits) {
    const int64_t s = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (s >= p.slots) return;
    const uint16_t vbits = static_cast<const uint16_t*>(p.MAPV)[s];
    if ((vbits & 0x7fffu) == 0) return;  // +-0: padding or an explicit zero, contributes nothing
    if (vbits != one_bits) *o.nonunit = 1;
    const int64_t cell = (int64_t)p.MAPZ[s / p.g] * o.Xp + p.MAPX[s];
    if (atomicCAS(&o.tabY[cell], -1, p.MAPY[s]) == -1)
        o.tabV[cell] = vbits;
    else
        o.ovf[atomicAdd(o.ovf_count, 1)] = (int32_t)s;
}

__global__ void weight_transpose(const uint16_t* __restrict__ W, OsParams o) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= o.Z * o.Mp * o.Cp) return;
    const int64_t c = i % o.Cp, m = (i / o.Cp) % o.Mp, z = i / (o.Cp * o.Mp);
    o.Wt[i] = (c < o.C && m < o.M) ? W[(z * o.C + c) * o.M + m] : (uint16_t)0;
}

// LDS position of 16-byte chunk ch of weight row n (CH chunks per row): the XOR spreads the rows
// that one 16-lane read phase touches over all banks.
template <int CH>
__device__ inline int swizzled_chunk(int n, int ch) {
    if constexpr (CH >= 16) return ch ^ (n % 16);
    else return ch ^ ((n / (16 / CH)) % CH);
}

// Two variants are launched for every call and one of them returns at once, according to the
// flag table_build leaves behind (the host never waits for it):
//   UNIT   every nonzero map value is 1, as in a plain convolution: the k-steps accumulate
//          straight into the running sums, which leaves registers for NT = 4 column blocks, so
//          the rows of an offset are gathered once for 128 output channels.  The fragments of
//          absent input points are replaced by zeros before they are used.
//   !UNIT  general values: NT = 2 and a separate accumulator per offset, scaled by the values.
// (the general variant with KS = 16 is built for one wavefront per SIMD: it needs all 256 registers)
template <typename T, int KS, int NT, bool UNIT, int WV, int RT>
__global__ __launch_bounds__(64 * WV, KS == 16 ? 1 : 2) void spconv_os(OsParams p) {
    // WV wavefronts, each with RT row tiles of 32 output points
    constexpr int THREADS = 64 * WV, ROWS = 32 * WV * RT;
    if ((*p.nonunit != 0) == UNIT) return;   // the other variant runs
    constexpr int CH = 2 * KS;             // 16-byte chunks per weight row
    constexpr int ROWB = CH * 16;          // bytes per weight row in LDS
    constexpr int TILE_CHUNKS = 32 * NT * CH;
    constexpr int PER_THREAD = TILE_CHUNKS / THREADS;
    constexpr int ROWS_PER_ROUND = THREADS / CH;    // weight rows staged by one round of all threads
    static_assert(TILE_CHUNKS % THREADS == 0 && THREADS % CH == 0, "staging assignment");
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][32 * NT * ROWB];

    // ids that share id % 8 run on one XCD: give the m-tiles of an x-block to the same one
    const int64_t q = blockIdx.x / 8, xcd = blockIdx.x % 8;
    const int64_t xblk = (q / p.m_tiles) * 8 + xcd;
    const int mt = (int)(q % p.m_tiles);
    if (xblk >= p.x_blocks) return;   // whole work-group leaves before any barrier

    const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
    const int half = lane / 32, l32 = lane % 32;
    const int m0 = mt * 32 * NT;
    const int ksteps = (int)((p.C + 15) / 16);
    const bool odd = p.C % 16 == 8;   // the last k-step holds 8 channels only
    const uint16_t* const In = static_cast<const uint16_t*>(p.In);

    // Offsets are visited cyclically from a start that differs between work-groups.
    const int Z = (int)p.Z;
    const int z_start = (int)((xblk * 7 + mt * 3) % Z);
    auto next_z = [&](int z) { return z + 1 == Z ? 0 : z + 1; };

    // Table cells of this lane's output points: row tile rt is 32 cells further on.
    const int64_t x_first = xblk * ROWS + wv * (32 * RT);
    const int32_t* const tab_y = p.tabY + (x_first + l32);
    const uint16_t* const tab_v = p.tabV + (x_first + l32);

    // Weight staging: thread owns chunk tid % CH of rows tid / CH + ROWS_PER_ROUND j.
    const int st_n = tid / CH, st_ch = tid % CH;
    const uint16_t* const w_src = p.Wt + ((int64_t)(m0 + st_n) * p.Cp + st_ch * 8);
    const int64_t w_round = (int64_t)ROWS_PER_ROUND * p.Cp;   // elements between a thread's chunks
    const int64_t w_next = p.Mp * p.Cp;                       // elements between offsets
    // (the loads of an iteration are issued unconditionally, wrapping around at the end of the
    // loop: with a fixed number of loads per iteration the compiler's wait counts let older
    // loads be consumed while newer ones are in flight)
    auto stage_load_one = [&](u32x4 (&reg)[PER_THREAD], int z, int j) {
        reg[j] = *reinterpret_cast<const u32x4*>(w_src + z * w_next + j * w_round);
    };
    auto stage_store = [&](int buf, const u32x4 (&reg)[PER_THREAD]) {
#pragma unroll
        for (int j = 0; j < PER_THREAD; ++j) {
            const int n = st_n + ROWS_PER_ROUND * j;
            *reinterpret_cast<u32x4*>(&lds[buf][n * ROWB + swizzled_chunk<CH>(n, st_ch) * 16]) = reg[j];
        }
    };
    // A fragments: k-step ks needs channels 16 ks + 8 (lane / 32) + [0, 8) of the lane's row.
    // Every lane always loads (no divergent or data-dependent branch between the loads, so the
    // compiler can count exactly how many are in flight).  A lane without an input point reads
    // the row of another lane of its quad (the texture addresser works through a load one
    // 64-byte piece per lane quad at a time, so this costs nothing extra), or row 0 when the
    // whole quad is absent; what it loaded is then replaced by zeros (UNIT) or multiplied by a
    // zero value later (!UNIT).  A k-step past C (weights are zero there) re-reads the last real
    // one; when the last real k-step holds 8 channels, both lane halves read those.
    const uint32_t full_h = (uint32_t)half * 8u, tail_h = odd ? 0u : full_h;
    auto gather_row = [&](int32_t y) {   // element offset of the row this lane loads from
        // largest y of the lane's quad: quad_perm [1,0,3,2] then [2,3,0,1]
        int32_t yq = max(y, __builtin_amdgcn_update_dpp(y, y, 0xB1, 0xF, 0xF, false));
        yq = max(yq, __builtin_amdgcn_update_dpp(yq, yq, 0x4E, 0xF, 0xF, false));
        return (uint32_t)max(y >= 0 ? y : yq, 0) * (uint32_t)p.ld_in;
    };
    auto gather_one = [&](int32_t y, uint32_t row, int ks) {
        const int kk = min(ks, ksteps - 1);   // uniform
        const uint32_t off = (uint32_t)kk * 16u + (kk == ksteps - 1 ? tail_h : full_h);
        const u32x4 raw = *reinterpret_cast<const u32x4*>(In + (uint64_t)row + off);
        const u32x4 zero = {0u, 0u, 0u, 0u};
        return __builtin_bit_cast(i16x8, (UNIT && y < 0) ? zero : raw);
    };
    auto table = [&](int32_t (&y)[RT], uint16_t (&vbits)[RT], int z) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            y[rt] = tab_y[z * p.Xp + rt * 32];
            vbits[rt] = tab_v[z * p.Xp + rt * 32];   // unspecified where y < 0
        }
    };

    f32x16 total[RT][NT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int ni = 0; ni < NT; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) total[rt][ni][r] = 0.f;

    u32x4 wreg[PER_THREAD];
    // Software pipeline.  One set of A fragments: the fragment of k-step ks is requested for the
    // next offset right after the MFMAs that read it for this one, so rows and weights run one
    // offset ahead and table cells two.  (Loads here mostly hit the L2, a few hundred clocks
    // away; an iteration lasts several thousand.)  The table load is issued first in an
    // iteration: the next iteration needs it first, and the load counter is in order.
    i16x8 a[RT][KS];
    int32_t y0[RT], y1[RT], y2[RT];
    uint16_t v0[RT], v1[RT], v2[RT];   // value bits; converted where they are used
    // Z >= 1 here.  zw / zt: the offsets whose weights and table cells are requested next.
    int zw = z_start, zt = z_start;
#pragma unroll
    for (int j = 0; j < PER_THREAD; ++j) stage_load_one(wreg, zw, j);
    zw = next_z(zw);
    table(y0, v0, zt), zt = next_z(zt);
    table(y1, v1, zt), zt = next_z(zt);
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const uint32_t row = gather_row(y0[rt]);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) a[rt][ks] = gather_one(y0[rt], row, ks);
    }
    stage_store(0, wreg);
    __syncthreads();

    // byte offset of this lane's B fragment for k-step 0, column block 0, inside a buffer
    const int b_row = l32 * ROWB;
    constexpr int W_EVERY = KS / PER_THREAD;   // k-steps between two weight loads
    static_assert(KS % PER_THREAD == 0, "weight loads spread over the k-steps");

    const int iterations = Z;
    for (int i = 0; i < iterations; ++i) {
        const int buf = i & 1;
        table(y2, v2, zt), zt = next_z(zt);      // iteration i + 2
        int32_t y_fill[RT];
        uint32_t row_fill[RT];
        bool present[RT];
        bool any = false;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            y_fill[rt] = i + 1 < Z ? y1[rt] : -1;   // nothing past the last iteration
            row_fill[rt] = gather_row(y_fill[rt]);
            present[rt] = y0[rt] >= 0;
            any |= __ballot(present[rt]) != 0;      // some output point of this wavefront has offset z
        }
        auto b_frag = [&](int ks, int ni) {
            const int pos = swizzled_chunk<CH>(l32, ks * 2 + half) * 16;   // 32 | ni * 32: same swizzle
            return *reinterpret_cast<const i16x8*>(&lds[buf][ni * 32 * ROWB + b_row + pos]);
        };
        // Rows and weights of iteration i + 1 are requested between the k-steps, one or two
        // loads after every group of MFMAs.
        auto loads_of_step = [&](int ks) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) a[rt][ks] = gather_one(y_fill[rt], row_fill[rt], ks);
            if (ks % W_EVERY == 0) stage_load_one(wreg, zw, ks / W_EVERY);
            __builtin_amdgcn_sched_barrier(0);
        };
        // every k-step up to 16 KS runs: weights past C are zero in LDS
        if constexpr (UNIT) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (any) {
#pragma unroll
                    for (int ni = 0; ni < NT; ++ni) {
                        const i16x8 b = b_frag(ks, ni);
#pragma unroll
                        for (int rt = 0; rt < RT; ++rt) total[rt][ni] = mfma32<T>(a[rt][ks], b, total[rt][ni]);
                    }
                }
                loads_of_step(ks);
            }
        } else {
            static_assert(UNIT || RT == 1, "general values: one row tile per wavefront");
            f32x16 acc[NT];
#pragma unroll
            for (int ni = 0; ni < NT; ++ni)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[ni][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (any) {
#pragma unroll
                    for (int ni = 0; ni < NT; ++ni) acc[ni] = mfma32<T>(a[0][ks], b_frag(ks, ni), acc[ni]);
                }
                loads_of_step(ks);
            }
            if (any) {
                const float v_row = present[0] ? half_bits_to_float(v0[0], T{}) : 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float vr = __shfl(v_row, 8 * (r / 4) + 4 * half + (r % 4));
#pragma unroll
                    for (int ni = 0; ni < NT; ++ni) total[0][ni][r] = fmaf(vr, acc[ni][r], total[0][ni][r]);
                }
            }
        }
        zw = next_z(zw);
        stage_store(buf ^ 1, wreg);
        __syncthreads();
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
            y0[rt] = y1[rt], v0[rt] = v1[rt], y1[rt] = y2[rt], v1[rt] = v2[rt];
    }

    // accumulator register r: output point 8 (r / 4) + 4 (lane / 32) + r % 4 of the row tile,
    // output channel m0 + 32 ni + lane % 32
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t x = x_first + rt * 32 + 8 * (r / 4) + 4 * half + (r % 4);
            if (x < p.X) {
#pragma unroll
                for (int ni = 0; ni < NT; ++ni) {
                    const int64_t m = m0 + ni * 32 + l32;
                    if (m < p.M) {
                        float* out = p.Out + x * p.ld_out + m;
                        *out = p.accumulate ? *out + total[rt][ni][r] : total[rt][ni][r];
                    }
                }
            }
        }
    }
}

// Contributions of the slots that lost their table cell: one work-group per slot (strided),
// one thread per output channel, fp32 atomics.  Runs after spconv_os has stored Out.
template <typename T>
__global__ __launch_bounds__(256) void spconv_overflow(ConvParams p, OsParams o) {
    const int32_t count = *o.ovf_count;
    const T* In = static_cast<const T*>(p.In);
    const T* W = static_cast<const T*>(p.W);
    const T* V = static_cast<const T*>(p.MAPV);
    for (int32_t e = blockIdx.x; e < count; e += gridDim.x) {
        const int64_t s = o.ovf[e];
        const float v = to_float(V[s]);
        const T* in = In + (int64_t)p.MAPY[s] * p.ld_in;
        const T* w = W + (int64_t)p.MAPZ[s / p.g] * p.C * p.M;
        for (int64_t m = threadIdx.x; m < p.M; m += 256) {
            float acc = 0.f;
            for (int64_t c = 0; c < p.C; ++c) acc = fmaf(to_float(in[c]), to_float(w[c * p.M + m]), acc);
            unsafeAtomicAdd(p.Out + (int64_t)p.MAPX[s] * p.ld_out + m, v * acc);
        }
    }
}

struct OsLayout {   // workspace carving for the output-stationary schedule
    int64_t Xp, Mp;
    int32_t Cp;
    size_t off_tabY, off_tabV, off_wt, off_count, off_ovf, bytes;
};

inline int ks_for(int64_t C) { return C <= 32 ? 2 : C <= 64 ? 4 : C <= 128 ? 8 : 16; }

OsLayout os_layout(int64_t X, int64_t Z, int64_t C, int64_t M, int64_t slots) {
    OsLayout L;
    L.Xp = ceil_div(X, 512) * 512;
    L.Mp = ceil_div(M, 128) * 128;
    L.Cp = 16 * ks_for(C);
    size_t b = 256;   // slack for aligning the caller's pointer
    // what depends on the map only comes first, so that calls with other channel counts find it
    // at the same place (reuse_map_tables)
    L.off_tabY = b, b += align_up((size_t)(Z * L.Xp) * 4, 256);
    L.off_tabV = b, b += align_up((size_t)(Z * L.Xp) * 2, 256);
    L.off_count = b, b += 256;   // overflow counter, non-unit flag
    L.off_ovf = b, b += align_up((size_t)std::max<int64_t>(slots, 1) * 4, 256);
    L.off_wt = b, b += align_up((size_t)(Z * L.Mp * L.Cp) * 2, 256);
    L.bytes = b;
    return L;
}

// The schedule pays off when an offset reaches a few of every 32 output points; below that
// most of its passes would be empty and the scatter kernel is used.
bool os_shape_ok(int64_t X, int64_t Z, int64_t C, int64_t M, int64_t slots, insum_dtype dt) {
    // (row offsets into In are 32-bit element counts: checked by the caller, which knows Y and ld_in)
    if (dt == INSUM_F32 || C % 8 != 0 || C < 8 || C > 256 || X <= 0 || Z <= 0 || M <= 0) return false;
    // sizes first, so that the products below stay far inside 64 bits
    if (X >= (1LL << 31) || Z >= (1LL << 20) || M >= (1LL << 24) || slots >= (1LL << 31)) return false;
    return slots * 16 >= X * Z && Z * (ceil_div(X, 512) * 512) < (1LL << 38) &&
           Z * (ceil_div(M, 128) * 128) * 256 < (1LL << 38) &&
           ceil_div(X, 128) * ceil_div(M, 64) + 8 * ceil_div(M, 64) < (1LL << 31);
}

template <typename T, int KS, int NT, bool UNIT, int WV, int RT>
void launch_os_variant(OsParams o, hipStream_t s) {
    o.m_tiles = (int32_t)ceil_div(o.M, 32 * NT);
    o.x_blocks = (int32_t)ceil_div(o.X, 32 * WV * RT);
    const unsigned grid = (unsigned)(ceil_div(o.x_blocks, 8) * 8 * o.m_tiles);
    hipLaunchKernelGGL((spconv_os<T, KS, NT, UNIT, WV, RT>), dim3(grid), dim3(64 * WV), 0, s, o);
}

template <typename T, int KS>
void launch_os_both(const OsParams& o, hipStream_t s) {
    // UNIT with KS <= 8 fits two wavefronts per SIMD: eight wavefronts (256 output points) share
    // one staged weight tile, which halves the weight traffic per MFMA (5 % faster than four).
    // RT = 2 (two row tiles per wavefront share every B fragment: half the LDS reads) was measured
    // too: 4 % slower at 256 registers, so one row tile it is.
    launch_os_variant<T, KS, (KS == 16 ? 2 : 4), true, (KS == 16 ? 4 : 8), 1>(o, s);
    launch_os_variant<T, KS, 2, false, 4, 1>(o, s);
}

template <typename T>
void launch_os(const ConvParams& p, const OsParams& o, bool reuse_map_tables, hipStream_t s) {
    const uint16_t one_bits = sizeof(T) == 2 && std::is_same<T, __half>::value ? 0x3C00 : 0x3F80;
    if (!reuse_map_tables) {
        hipLaunchKernelGGL(table_fill, dim3((unsigned)ceil_div(o.Z * o.Xp, 256)),
                           dim3(256), 0, s, o);
        hipLaunchKernelGGL(table_build, dim3((unsigned)ceil_div(p.slots, 256)), dim3(256), 0, s, p, o, one_bits);
    }
    hipLaunchKernelGGL(weight_transpose, dim3((unsigned)ceil_div(o.Z * o.Mp * o.Cp, 256)), dim3(256), 0, s,
                       static_cast<const uint16_t*>(p.W), o);
    switch (o.Cp / 16) {
        case 2: launch_os_both<T, 2>(o, s); break;
        case 4: launch_os_both<T, 4>(o, s); break;
        case 8: launch_os_both<T, 8>(o, s); break;
        default: launch_os_both<T, 16>(o, s); break;
    }
    hipLaunchKernelGGL(spconv_overflow<T>, dim3(256), dim3(256), 0, s, p, o);
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

extern "C" size_t insum_spconv_groupcoo_workspace_bytes(int64_t X, int64_t Z, int64_t C, int64_t M,
                                                        int64_t G, int32_t g, insum_dtype dt) {
    if (X < 0 || Z < 0 || C < 0 || M < 0 || G < 0 || g <= 0 || !dtype_valid(dt)) return 0;
    if (G >= (1LL << 31)) return 0;   // (also keeps G * g inside 64 bits)
    const int64_t slots = G * (int64_t)g;
    if (!os_shape_ok(X, Z, C, M, slots, dt)) return 0;
    return os_layout(X, Z, C, M, slots).bytes;
}

extern "C" insum_status insum_spconv_groupcoo(int64_t X, int64_t Y, int64_t Z, int64_t C, int64_t M,
                                              int64_t G, int32_t g, const int32_t* MAPZ,
                                              const int32_t* MAPX, const int32_t* MAPY, const void* MAPV,
                                              const void* In, int64_t ld_in, const void* W, insum_dtype dt,
                                              float* Out, int64_t ld_out, int accumulate,
                                              int reuse_map_tables, void* workspace,
                                              size_t workspace_bytes, void* stream) {
    if (X < 0 || Y < 0 || Z < 0 || C < 0 || M < 0 || G < 0 || g <= 0) return INSUM_ERR_INVALID_ARG;
    if (X >= (1LL << 31) || Y >= (1LL << 31) || Z >= (1LL << 31) || C >= (1LL << 31) || M >= (1LL << 31))
        return INSUM_ERR_INVALID_ARG;
    if (!dtype_valid(dt) || ld_in < C || ld_out < M) return INSUM_ERR_INVALID_ARG;
    if (G >= (1LL << 31) || G * (int64_t)g >= (1LL << 40)) return INSUM_ERR_INVALID_ARG;
    if (X > 0 && M > 0 && !Out) return INSUM_ERR_INVALID_ARG;
    if (G > 0 && (!MAPZ || !MAPX || !MAPY || !MAPV)) return INSUM_ERR_INVALID_ARG;
    if (G > 0 && C > 0 && M > 0 && (!In || !W)) return INSUM_ERR_INVALID_ARG;
    if (G > 0 && (X == 0 || Y == 0 || Z == 0)) return INSUM_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (X == 0 || M == 0) return INSUM_OK;

    ConvParams p;
    p.X = X, p.Y = Y, p.C = C, p.M = M;
    p.slots = G * (int64_t)g;
    p.g = g;
    p.MAPZ = MAPZ, p.MAPX = MAPX, p.MAPY = MAPY, p.MAPV = MAPV;
    p.In = In, p.ld_in = ld_in, p.W = W, p.Out = Out, p.ld_out = ld_out;
    p.tiles = ceil_div(p.slots, 32);
    p.waves_total = 0;
    const bool rows_ok = ld_in % 8 == 0 && reinterpret_cast<uintptr_t>(In) % 16 == 0;

    if (G > 0 && rows_ok && Y * ld_in < (1LL << 32) && os_shape_ok(X, Z, C, M, p.slots, dt)) {
        const OsLayout L = os_layout(X, Z, C, M, p.slots);
        if (!workspace || workspace_bytes < L.bytes) return INSUM_ERR_CAPACITY;
        char* base = reinterpret_cast<char*>((reinterpret_cast<uintptr_t>(workspace) + 255) / 256 * 256) - 256;
        OsParams o;
        o.X = X, o.Z = Z, o.C = C, o.M = M, o.Xp = L.Xp, o.Mp = L.Mp, o.Cp = L.Cp;
        o.tabY = reinterpret_cast<int32_t*>(base + L.off_tabY);
        o.tabV = reinterpret_cast<uint16_t*>(base + L.off_tabV);
        o.Wt = reinterpret_cast<uint16_t*>(base + L.off_wt);
        o.ovf_count = reinterpret_cast<int32_t*>(base + L.off_count);
        o.nonunit = o.ovf_count + 1;
        o.ovf = reinterpret_cast<int32_t*>(base + L.off_ovf);
        o.In = In, o.ld_in = ld_in, o.Out = Out, o.ld_out = ld_out, o.accumulate = accumulate ? 1 : 0;
        o.m_tiles = 0;   // set per variant
        o.x_blocks = 0;  // set per variant
        if (dt == INSUM_F16) launch_os<__half>(p, o, reuse_map_tables != 0, s);
        else launch_os<bf16_t>(p, o, reuse_map_tables != 0, s);
        INSUM_HIP_TRY(hipGetLastError());
        return INSUM_OK;
    }

    if (!accumulate) {
        const int64_t n = X * M;
        if (ceil_div(n, 256) >= (1LL << 31)) return INSUM_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(fill_zero_rows, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s, Out, X, M, ld_out);
    }
    if (G > 0 && C > 0) {
        const bool mfma_ok = dt != INSUM_F32 && C % 8 == 0 && C >= 8 && C <= 256 && rows_ok &&
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
