// SpMM over BlockGroupCOO for gfx950:
//     C[AM[p]*bM + bm, n] (+)= sum_{q,bk} AV[p,q,bm,bk] * B[AK[p,q]*bK + bk, n]
// (paper: Section 4.1, BlockGroupCOO Einsum; the fused gather - dot - scatter structure of
// the generated kernel in Section 5.2: the whole reduction of an output tile stays on chip
// and the tile is written once).
//
// MFMA kernel
//   * One workgroup owns one block row x NT output columns (NT = 64 per wavefront); each
//     wavefront keeps its bM x 64 fp32 accumulator in registers for the whole block row,
//     so C is written exactly once and never needs atomics.  The groups of a block row are
//     consecutive in AM (non-decreasing); the workgroup finds them by binary search.  A
//     block row without groups just writes zeros.
//   * Work is cut into steps: one stored block (padding blocks repeat the previous block
//     column and are skipped) x one k-chunk of KC rows.  Per step the gathered B tile
//     (KC x NT) and the A chunk (bM x KC) are copied global -> LDS by the DMA path
//     (global_load_lds_dwordx4: 16 bytes per lane, no VGPR staging) into a ring of S
//     stages; S-1 stages are in flight while one is consumed, with one barrier per step.
//   * The DMA writes lane i of an instruction to LDS slot i (16-byte units), but each lane
//     may read any global address, so the LDS layout is chosen by permuting the sources.
//     The L1 handles one aligned 64-byte piece per 4 adjacent lanes per clock (measured:
//     21 clk for a contiguous 1 KiB instruction, 70 clk when every lane sits in another
//     line), so every lane quad reads 64 contiguous bytes:
//       - B: quads ordered [k/4][n/32][k%4], a quad = 32 columns of one row.  The
//         4(k) x 16(n) patch that a 16-lane group fetches with the transposing read
//         ds_read_b64_tr_b16 is four 32-byte pieces 64 bytes apart, and the two patches of
//         a 32-lane half fill a 256-byte window exactly (no bank conflicts).  The read
//         returns 4 consecutive k of one column per lane - the MFMA operand layout -
//         although B is row-major.
//       - A: row-major, a quad = the 32 k-values (64 bytes) of one row, its four units
//         stored in the order j ^ ((row/4) % 4) so that the 16 lanes of a fragment read
//         (rows 64 bytes apart) fall into 16 different bank groups.
//   * v_mfma_f32_32x32x16_{bf16,f16} is issued with the B fragment as first operand, i.e.
//     it produces the transposed tile: a lane ends up with 4 consecutive columns of one
//     output row per register quad, which are packed and stored as 8 (16-bit C) or 16
//     (fp32 C) contiguous bytes.
//   * LDS reads are issued as inline assembly with explicit s_waitcnt: the compiler would
//     otherwise wait for every outstanding DMA load before each LDS read, which would
//     serialise the ring.  DMA loads are never skipped or masked (ragged column tiles clamp
//     the address instead), so the number of outstanding loads per stage is constant and
//     s_waitcnt vmcnt(n) identifies a stage exactly.
//   * Workgroup ids are mapped so that the workgroups an XCD receives (id % 8) share
//     column tiles: the B columns an XCD touches are a 1/8 .. 1/1 slice that its L2 can
//     hold or mostly hold.
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
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

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

// First index i in the non-decreasing array a[0..n) with a[i] >= v, found by the whole
// wavefront: every round probes 64 evenly spaced positions with one load and narrows the
// range by a factor of 64 (two rounds for n <= 4096 instead of twelve dependent loads).
__device__ inline int64_t wave_lower_bound(const int32_t* __restrict__ a, int64_t n, int32_t v, int lane) {
    int64_t lo = 0, hi = n;  // a[i] < v for i < lo, a[i] >= v for i >= hi
    while (lo < hi) {
        const int64_t step = (hi - lo + 63) / 64;
        const int64_t idx = lo + (int64_t)lane * step;
        const bool less = idx < hi && a[idx] < v;
        const int c = __popcll(__ballot(less));  // probes 0..c-1 are < v (a is monotone)
        const int64_t first_ge = lo + (int64_t)c * step;  // probe c, if it exists, is >= v
        if (c > 0) lo = lo + (int64_t)(c - 1) * step + 1;
        if (first_ge < hi) hi = first_ge;
    }
    return lo;
}

// Walks the stored blocks of one block row, k-chunk by k-chunk, skipping padding blocks
// (a padding block repeats the block column of the slot before it in the same group).
// Sixty-four slots at a time are read with one coalesced load; which of them are stored
// blocks is a 64-bit mask, and stepping to the next block is scalar bit arithmetic plus
// a v_readlane - no memory access, so the DMA ring is never drained to wait for an index.
struct RowIter {
    const int32_t* AK;
    int64_t base, slot_end;  // flat slot index p*g+q of lane 0; end of the block row
    int64_t row_base;        // first slot of the block row (a multiple of g)
    int32_t g, kchunks, kc;
    int32_t ak;              // per lane: AK[base + lane]
    uint64_t mask;           // stored blocks of this batch not yet visited
    int32_t cur;             // lane of the current block
    bool has;

    __device__ void load_batch(int lane) {
        has = false;
        while (base < slot_end) {
            const int64_t idx = base + lane;
            const bool ok = idx < slot_end;
            const int32_t c = ok ? AK[idx] : -1;
            const int32_t prev = (ok && ((uint32_t)(idx - row_base) % (uint32_t)g) != 0) ? AK[idx - 1] : -2;
            ak = c;
            mask = __ballot(ok && c != prev);
            if (mask) {
                cur = __builtin_ctzll(mask);
                has = true;
                return;
            }
            base += 64;
        }
    }
    __device__ int32_t col() const { return __builtin_amdgcn_readlane(ak, cur); }
    __device__ int64_t slot() const { return base + cur; }
    __device__ void next(int lane) {
        if (++kc < kchunks) return;
        kc = 0;
        mask &= mask - 1;
        if (mask) {
            cur = __builtin_ctzll(mask);
        } else {
            base += 64;
            load_batch(lane);
        }
    }
};

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding: vmcnt in bits
// 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8).
template <int N>
__device__ inline void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;

// How workgroup ids map to (block row, column tile); see the header comment.
struct TileMap {
    int32_t mode;  // 0: tile fastest; 1: ntiles % 8 == 0; 2: 8 % ntiles == 0
    int32_t ntiles;
    int64_t nrows;
    __device__ bool get(int64_t id, int64_t& row, int32_t& tile) const {
        if (mode == 1) {
            const int32_t tp = ntiles / 8;
            const int64_t j = id / 8;
            tile = (int32_t)(id % 8) + 8 * (int32_t)(j % tp);
            row = j / tp;
        } else if (mode == 2) {
            const int32_t x = (int32_t)(id % 8);
            tile = x % ntiles;
            row = (id / 8) * (8 / ntiles) + x / ntiles;
        } else {
            tile = (int32_t)(id % ntiles);
            row = id / ntiles;
        }
        return row < nrows;
    }
};

// DMA instructions of one stage that wavefront W issues (W is a template parameter so that
// the split between B and A instructions and all offsets are resolved at compile time).
// Sources are "uniform base + 32-bit lane offset", which maps onto the SGPR-base
// addressing mode of global_load_lds: two scalar adds and one M0 write per instruction.
template <int W, int WAVES, int BM>
__device__ inline void issue_stage(const char* b_step, const char* a_step,
                                   const uint32_t (&b_lane)[WAVES / 2], uint32_t a_lane,
                                   int64_t b_kq_stride, int64_t a_instr_stride, char* stage) {
    constexpr int NT = WAVES * 64;
    constexpr int B_INSTR = 8 * (NT / 128);
    constexpr int STAGE_INSTR = B_INSTR + BM / 16;
    constexpr int LPW = (STAGE_INSTR + WAVES - 1) / WAVES;
#pragma unroll
    for (int j = 0; j < LPW; ++j) {
        const int idx = (W * LPW + j < STAGE_INSTR) ? W * LPW + j : STAGE_INSTR - 1;  // duplicates reload the same bytes
        const char* src;
        if (idx < B_INSTR) src = b_step + (idx / (NT / 128)) * b_kq_stride + b_lane[idx % (NT / 128)];
        else src = a_step + (idx - B_INSTR) * a_instr_stride + a_lane;
        __builtin_amdgcn_global_load_lds((global_void_ptr)src, (lds_void_ptr)(stage + idx * 1024), 16, 0, 0);
    }
}

template <typename T, typename TC, int BM, int KC, int WAVES, int S>
__global__ __launch_bounds__(WAVES * 64) void spmm_block_mfma(BlockParams p, TileMap map) {
    constexpr int NT = WAVES * 64;   // output columns per workgroup
    constexpr int MI = BM / 32;      // 32-row MFMA tiles per block
    constexpr int KS = KC / 16;      // MFMA k-steps per chunk
    constexpr int NI = 2;            // 32-column MFMA tiles per wavefront
    static_assert(KC == 32, "a lane quad moves the 32 k-values (64 bytes) of one A row");
    constexpr int B_INSTR = (KC / 4) * (NT / 128);  // DMA instructions (1 KiB each) per B tile
    constexpr int A_INSTR = BM / 16;                // ... per A chunk (16 rows each)
    constexpr int STAGE_INSTR = B_INSTR + A_INSTR;
    constexpr int LPW = (STAGE_INSTR + WAVES - 1) / WAVES;  // DMA instructions per wave and stage
    constexpr int STAGE_BYTES = STAGE_INSTR * 1024;
    static_assert((WAVES == 2 || WAVES == 4 || WAVES == 8) && S >= 2 && (S - 2) * LPW < 64, "unsupported tiling");
    __shared__ __attribute__((aligned(1024))) char lds[S * STAGE_BYTES];

    int64_t brow;
    int32_t tile;
    if (!map.get(blockIdx.x, brow, tile)) return;

    const int tid = threadIdx.x;
    const int lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int64_t ntile0 = (int64_t)tile * NT;

    const int64_t p0 = wave_lower_bound(p.AM, p.G, (int32_t)brow, lane);
    const int64_t p1 = wave_lower_bound(p.AM, p.G, (int32_t)brow + 1, lane);

    RowIter ld;
    ld.AK = p.AK;
    ld.base = p0 * p.g;
    ld.row_base = p0 * p.g;
    ld.slot_end = p1 * p.g;
    ld.g = p.g;
    ld.kc = 0;
    ld.kchunks = p.bK / KC;
    ld.load_batch(lane);

    // ---- DMA addressing (per lane, fixed for the whole kernel) ----
    // B instruction j: rows 4*(j / (NT/128)) .. +3, column groups 4*(j % (NT/128)) .. +3;
    // quad q = lane/4 -> row q%4, column group q/4; lane%4 -> 8 columns of the quad's 32.
    // A ragged column tile clamps the column (the DMA is never skipped or masked).
    const int quad = lane / 4;
    const int64_t ldb_bytes = p.ldb * 2;
    uint32_t b_lane[NT / 128];
#pragma unroll
    for (int half = 0; half < NT / 128; ++half) {
        int64_t n = ntile0 + 128 * half + 32 * (quad / 4) + 8 * (lane % 4);
        if (n > p.N - 8) n = p.N - 8;
        b_lane[half] = (uint32_t)((quad % 4) * ldb_bytes + n * 2);
    }
    // A instruction a: rows 16*a .. +15; quad -> row, lane%4 -> unit (lane%4) ^ ((row/4)%4)
    const uint32_t a_lane_src = (uint32_t)((quad * p.bK + 8 * ((lane % 4) ^ ((quad / 4) % 4))) * 2);
    const int64_t b_kq_stride = 4 * ldb_bytes;
    const int64_t a_instr_stride = 16 * (int64_t)p.bK * 2;
    const int64_t block_bytes = (int64_t)p.bM * p.bK * 2;
    const char* const Bb = static_cast<const char*>(p.B);
    const char* const Ab = static_cast<const char*>(p.AV);

    auto issue = [&](const RowIter& s, int buf) {
        const char* b_step = Bb + ((int64_t)s.col() * p.bK + s.kc * KC) * ldb_bytes;
        const char* a_step = Ab + s.slot() * block_bytes + s.kc * KC * 2;
        char* stage = lds + buf * STAGE_BYTES;
#define INSUM_ISSUE_CASE(W)                                                                    \
    if constexpr (WAVES > W) {                                                                 \
        if (wave == W)                                                                         \
            issue_stage<W, WAVES, BM>(b_step, a_step, b_lane, a_lane_src, b_kq_stride,         \
                                      a_instr_stride, stage);                                  \
    }
        INSUM_ISSUE_CASE(0) INSUM_ISSUE_CASE(1) INSUM_ISSUE_CASE(2) INSUM_ISSUE_CASE(3)
        INSUM_ISSUE_CASE(4) INSUM_ISSUE_CASE(5) INSUM_ISSUE_CASE(6) INSUM_ISSUE_CASE(7)
#undef INSUM_ISSUE_CASE
    };

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    // ---- LDS read addressing ----
    // B element (k, n) of the tile sits at byte ((k/4 * NT/32 + n/32) * 4 + k%4) * 64 + (n%32) * 2.
    // Patch read: 16-lane group b = lane/16 -> column half nb = b%2, k half h = b/2; lane
    // s = lane%16 reads row s/4, columns 4*(s%4)..+3 of the patch.  Lane-dependent part:
    const int s16 = lane % 16;
    const int tr_base = (2 * (lane / 32) * (NT / 32) + 2 * wave) * 256 + (s16 / 4) * 64 +
                        (16 * ((lane / 16) % 2) + 4 * (s16 % 4)) * 2;
    // immediate part: ((4*ks + r) * (NT/32) + ni) * 256
    // A fragment (mi, ks): lane -> row m = 32*mi + lane%32, unit j = 2*ks + lane/32, stored at
    // m*64 + (j ^ ((m/4)%4))*16; (m/4)%4 does not depend on mi.
    const int a_swz = ((lane % 32) / 4) % 4;
    int a_lane[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) a_lane[ks] = (lane % 32) * 64 + (((2 * ks + lane / 32) ^ a_swz) * 16);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_void_ptr)lds;

    // Operand fragments of k-step ks are requested while the MFMAs of k-step ks-1 run
    // (two register sets); lgkmcnt counts LDS reads in order, so waiting until only the
    // reads of the next k-step are outstanding means the current ones have arrived.
    constexpr int READS = MI + 2 * NI;  // LDS reads per k-step and wavefront
    auto compute = [&](int buf) {
        const uint32_t sb = lds0 + buf * STAGE_BYTES;
        const uint32_t b_addr = sb + tr_base;
        i16x8 a[2][MI];
        i16x4 blo[2][NI], bhi[2][NI];
#pragma unroll
        for (int ks = 0; ks <= KS; ++ks) {
            if (ks < KS) {
                const int set = ks % 2;
                const uint32_t a_addr = sb + B_INSTR * 1024 + a_lane[ks];
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
                    asm volatile("ds_read_b128 %0, %1 offset:%2"
                                 : "=v"(a[set][mi]) : "v"(a_addr), "n"(mi * 2048) : "memory");
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2"
                                 : "=v"(blo[set][ni]) : "v"(b_addr), "n"(((4 * ks + 0) * (NT / 32) + ni) * 256) : "memory");
                    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2"
                                 : "=v"(bhi[set][ni]) : "v"(b_addr), "n"(((4 * ks + 1) * (NT / 32) + ni) * 256) : "memory");
                }
            }
            if (ks > 0) {
                const int set = (ks - 1) % 2;
                // The reads of k-step ks (if any) stay outstanding.  The empty statements tie
                // the fragment registers to the wait, so no MFMA that uses them moves above it.
                if (ks < KS) asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(READS) : "memory");
                else asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) asm volatile("" : "+v"(a[set][mi])::"memory");
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) asm volatile("" : "+v"(blo[set][ni]), "+v"(bhi[set][ni])::"memory");
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    const i16x8 b = __builtin_shufflevector(blo[set][ni], bhi[set][ni], 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi) acc[mi][ni] = mfma32<T>(b, a[set][mi], acc[mi][ni]);
                }
            }
        }
    };

    // ---- ring: stage j lives in buffer j % S ----
    int issued = 0;
#pragma unroll
    for (int j = 0; j < S - 1; ++j) {
        if (ld.has) {
            issue(ld, j);
            ld.next(lane);
            ++issued;
        }
    }
    int buf = 0, fill = S - 1;
    for (int i = 0; i < issued; ++i) {
        // Stage i has landed once at most the S-2 younger stages are outstanding; near the
        // end of the row fewer are in flight and everything is waited for.
        if (issued - i >= S - 1) wait_vmcnt<(S - 2) * LPW>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();   // everyone's part of stage i is in LDS; compute(i-1) done
        if (ld.has) {
            issue(ld, fill);
            ld.next(lane);
            ++issued;
        }
        compute(buf);
        buf = buf + 1 == S ? 0 : buf + 1;
        fill = fill + 1 == S ? 0 : fill + 1;
    }

    // ---- epilogue: acc holds the transposed tiles: lane -> output row lane%32 (+32*mi),
    // register quad q -> columns 32*ni + 8*q + 4*(lane/32) .. +3
    TC* C = static_cast<TC*>(p.C);
    const bool accumulate = p.accumulate != 0;
    if constexpr (sizeof(TC) == 2) {
        if (!accumulate) {
            // 16-bit C: round, park the wavefront's bM x 64 tile in LDS (the ring is idle now)
            // and write it out as full 128-byte row segments, 16 bytes per lane.
            constexpr int CSTRIDE = 144;  // bytes per staged row (128 of data)
            static_assert(WAVES * BM * CSTRIDE <= S * STAGE_BYTES, "C staging does not fit the ring");
            __builtin_amdgcn_s_barrier();  // the other wavefronts are done reading the ring
            char* cw = lds + wave * (BM * CSTRIDE);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        union {
                            TC h[4];
                            u32x2 u;
                        } pk;
#pragma unroll
                        for (int e = 0; e < 4; ++e) pk.h[e] = from_float<TC>(acc[mi][ni][4 * q + e]);
                        *reinterpret_cast<u32x2*>(cw + (32 * mi + lane % 32) * CSTRIDE +
                                                  (32 * ni + 8 * q + 4 * (lane / 32)) * 2) = pk.u;
                    }
            const int64_t col = ntile0 + 64 * wave + 8 * (lane % 8);
#pragma unroll
            for (int it = 0; it < BM / 8; ++it) {
                const int r = it * 8 + lane / 8;
                const u32x4 v = *reinterpret_cast<const u32x4*>(cw + r * CSTRIDE + (lane % 8) * 16);
                if (col < p.N)
                    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(C + (brow * BM + r) * p.ldc + col));
            }
            return;
        }
    }
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int64_t row = brow * BM + 32 * mi + lane % 32;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int64_t col = ntile0 + 64 * wave + 32 * ni + 8 * q + 4 * (lane / 32);
                if (col < p.N) {
                    TC* dst = C + row * p.ldc + col;
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = acc[mi][ni][4 * q + e];
                    if (accumulate) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += to_float(dst[e]);
                    }
                    if constexpr (sizeof(TC) == 4) {
                        *reinterpret_cast<f32x4*>(dst) = f32x4{v[0], v[1], v[2], v[3]};
                    } else {
                        union {
                            TC h[4];
                            u32x2 u;
                        } pk;
#pragma unroll
                        for (int e = 0; e < 4; ++e) pk.h[e] = from_float<TC>(v[e]);
                        *reinterpret_cast<u32x2*>(dst) = pk.u;
                    }
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

constexpr int kWaves = 4;   // wavefronts per workgroup -> 256 output columns
constexpr int kStages = 4;  // LDS ring depth

TileMap make_map(int64_t nrows, int64_t ntiles, int64_t& grid) {
    TileMap m;
    m.ntiles = (int32_t)ntiles;
    m.nrows = nrows;
    if (ntiles % 8 == 0) {
        m.mode = 1;
        grid = nrows * ntiles;
    } else if (8 % ntiles == 0) {
        m.mode = 2;
        grid = 8 * ceil_div(nrows, 8 / ntiles);
    } else {
        m.mode = 0;
        grid = nrows * ntiles;
    }
    return m;
}

template <typename T, typename TC, int BM>
void launch_mfma_kc(const BlockParams& p, hipStream_t s) {
    int64_t grid = 0;
    const TileMap map = make_map(p.M / p.bM, ceil_div(p.N, kWaves * 64), grid);
    hipLaunchKernelGGL((spmm_block_mfma<T, TC, BM, 32, kWaves, kStages>), dim3((unsigned)grid),
                       dim3(kWaves * 64), 0, s, p, map);
}

template <typename T, typename TC>
void launch_typed(const BlockParams& p, bool mfma_ok, hipStream_t s) {
    if constexpr (sizeof(T) == 2) {
        if (mfma_ok && p.bM == 32) return launch_mfma_kc<T, TC, 32>(p, s);
        if (mfma_ok && p.bM == 64) return launch_mfma_kc<T, TC, 64>(p, s);
        if (mfma_ok && p.bM == 128) return launch_mfma_kc<T, TC, 128>(p, s);
    }
    const dim3 grid((unsigned)(p.M / p.bM), (unsigned)ceil_div(p.N, 256));
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

    const bool mfma_ok = bK % 32 == 0 && N % 8 == 0 && N >= 8 && ldb % 8 == 0 && ldb < (1LL << 27) &&
                         ldc % (c_dt == INSUM_F32 ? 4 : 8) == 0 &&
                         (reinterpret_cast<uintptr_t>(C) % 16) == 0 &&
                         (M / bM) * ceil_div(N, 128) < (1LL << 31) - 8 &&
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
