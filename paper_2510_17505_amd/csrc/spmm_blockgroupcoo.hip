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
//     block row without groups just writes zeros.  (With a work plan - further down - a
//     block row much longer than the others is cut into chunks for several workgroups,
//     whose fp32 tiles the last one to finish adds in chunk order.)
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
#include <cstdlib>
#include <type_traits>

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

// ---- work plan (optional, kept in the caller's workspace) -------------------------------------
// insum_spmm_blockgroupcoo_plan cuts the block rows into work items - a whole block row, or,
// for a block row longer than about 5/4 of the mean load of a workgroup slot, equal chunks of
// its groups - and lists them longest first.  Workgroups are dispatched in id order, so the
// long items start first and the short ones fill the gaps (longest-processing-time-first list
// scheduling); without it a long block row that happens to start late is the tail of the launch.
// The chunks of a split row put their fp32 tiles into the workspace; the workgroup that
// arrives last (a counter per row and column tile) adds them in chunk order and writes C, so
// the result does not depend on timing.
constexpr uint64_t kPlanMagic = 0x314e414c504d5553ull;
constexpr int kPlanBuckets = 1024;

struct PlanHeader {
    uint64_t magic;
    int64_t G, nrows, n_items, n_split_rows, n_chunks;
    const int32_t* AM;
    int32_t g, bM, ntiles, nt, chunk_groups, reserved;
};

struct PlanItem {
    int32_t row, p0, p1;     // block row and its groups [p0, p1)
    int32_t split;           // -1: the item is a whole block row; else index of the split row
    int32_t chunk, nchunks;  // position among the chunks of that row
    int32_t first_part;      // index of the row's first partial tile set
    int32_t reserved;
};

struct PlanView {  // what the SpMM kernel needs of a planned workspace; hdr == nullptr: no plan
    const PlanHeader* hdr;
    const PlanItem* items;
    int32_t* counters;
    float* partials;
    int32_t chunk_groups;
};

// DMA instructions of one stage that wavefront W issues (W is a template parameter so that
// the split between B and A instructions and all offsets are resolved at compile time).
// Sources are "uniform base + 32-bit lane offset", which maps onto the SGPR-base
// addressing mode of global_load_lds: two scalar adds and one M0 write per instruction.
// Every wavefront issues the same number of instructions per stage (so that one s_waitcnt
// value identifies a stage in all of them); when the count does not divide, the last
// wavefront repeats the final instruction.  (Dealing 18 instructions out as 5+5+4+4 with
// per-wavefront wait counts measured 7 % slower on 32-row blocks than 4 x 5 with two repeats.)
template <int W, int WAVES, int NI, int BM>
__device__ inline void issue_stage(const char* b_step, const char* a_step,
                                   const uint32_t (&b_lane)[WAVES * NI / 4], uint32_t a_lane,
                                   int64_t b_kq_stride, int64_t a_instr_stride, char* stage) {
    constexpr int NT = WAVES * NI * 32;
    constexpr int B_INSTR = 8 * (NT / 128);
    constexpr int STAGE_INSTR = B_INSTR + BM / 16;
    constexpr int LPW = (STAGE_INSTR + WAVES - 1) / WAVES;
#pragma unroll
    for (int j = 0; j < LPW; ++j) {
        const int idx = (W * LPW + j < STAGE_INSTR) ? W * LPW + j : STAGE_INSTR - 1;  // repeats reload the same bytes
        const char* src;
        if (idx < B_INSTR) src = b_step + (idx / (NT / 128)) * b_kq_stride + b_lane[idx % (NT / 128)];
        else src = a_step + (idx - B_INSTR) * a_instr_stride + a_lane;
        __builtin_amdgcn_global_load_lds((global_void_ptr)src, (lds_void_ptr)(stage + idx * 1024), 16, 0, 0);
    }
}

template <typename T, typename TC, int BM, int WAVES, int NI, int S>
__global__ __launch_bounds__(WAVES * 64) void spmm_block_mfma(BlockParams p, TileMap map, PlanView plan) {
    constexpr int KC = 32;               // k-values per step: a lane quad moves the 64 bytes of one A row
    constexpr int NT = WAVES * NI * 32;  // output columns per workgroup
    constexpr int MI = BM / 32;          // 32-row MFMA tiles per block
    constexpr int KS = KC / 16;          // MFMA k-steps per step
    constexpr int B_INSTR = (KC / 4) * (NT / 128);  // DMA instructions (1 KiB each) per B tile
    constexpr int A_INSTR = BM / 16;                // ... per A chunk (16 rows each)
    constexpr int STAGE_INSTR = B_INSTR + A_INSTR;
    constexpr int LPW = (STAGE_INSTR + WAVES - 1) / WAVES;  // DMA instructions per wave and stage
    constexpr int STAGE_BYTES = STAGE_INSTR * 1024;
    static_assert((WAVES == 2 || WAVES == 4 || WAVES == 8) && (NI == 1 || NI == 2) && NT % 128 == 0 &&
                  S >= 2 && (S - 2) * LPW < 64, "unsupported tiling");
    __shared__ __attribute__((aligned(1024))) char lds[S * STAGE_BYTES];

    int64_t idx;
    int32_t tile;
    if (!map.get(blockIdx.x, idx, tile)) return;

    const int tid = threadIdx.x;
    const int lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int64_t ntile0 = (int64_t)tile * NT;
    const int64_t nrows = p.M / BM;

    // ---- which groups are mine: an item of the plan, or a whole block row found by search ----
    int64_t brow, p0, p1;
    int32_t split = -1, chunk = 0, nchunks = 1, first_part = 0;
    const PlanHeader* const h = plan.hdr;
    bool planned = false;
    PlanItem it{};
    if (h != nullptr) {
        it = plan.items[idx];   // idx < the capacity of the list; requested together with the header
        planned = h->magic == kPlanMagic && h->G == p.G && h->nrows == nrows && h->AM == p.AM && h->g == p.g &&
                  h->bM == BM && h->ntiles == map.ntiles && h->nt == NT && h->chunk_groups == plan.chunk_groups;
    }
    if (planned) {
        if (idx >= h->n_items) return;
        brow = it.row;
        p0 = it.p0;
        p1 = it.p1;
        split = it.split;
        chunk = it.chunk;
        nchunks = it.nchunks;
        first_part = it.first_part;
    } else {
        if (idx >= nrows) return;
        brow = idx;
        p0 = wave_lower_bound(p.AM, p.G, (int32_t)brow, lane);
        p1 = wave_lower_bound(p.AM, p.G, (int32_t)brow + 1, lane);
    }

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

    // Starts the copies of the iterator's current step (one stored block x KC values of k)
    // into buffer `buf` and moves the iterator on.
    int issued = 0;
    auto issue = [&](int buf) {
        const char* b_step = Bb + ((int64_t)ld.col() * p.bK + ld.kc * KC) * ldb_bytes;
        const char* a_step = Ab + ld.slot() * block_bytes + ld.kc * KC * 2;
        char* stage = lds + buf * STAGE_BYTES;
#define INSUM_ISSUE_CASE(W)                                                                    \
    if constexpr (WAVES > W) {                                                                 \
        if (wave == W)                                                                         \
            issue_stage<W, WAVES, NI, BM>(b_step, a_step, b_lane, a_lane_src, b_kq_stride,     \
                                          a_instr_stride, stage);                              \
    }
        INSUM_ISSUE_CASE(0) INSUM_ISSUE_CASE(1) INSUM_ISSUE_CASE(2) INSUM_ISSUE_CASE(3)
        INSUM_ISSUE_CASE(4) INSUM_ISSUE_CASE(5) INSUM_ISSUE_CASE(6) INSUM_ISSUE_CASE(7)
#undef INSUM_ISSUE_CASE
        ld.next(lane);
        ++issued;
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
    const int tr_base = (2 * (lane / 32) * (NT / 32) + NI * wave) * 256 + (s16 / 4) * 64 +
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
#pragma unroll
    for (int j = 0; j < S - 1; ++j) {
        if (ld.has) issue(j);
    }
    int buf = 0, fill = S - 1;
    for (int i = 0; i < issued; ++i) {
        // Stage i has landed once at most the S-2 younger stages are outstanding; near the
        // end of the row fewer are in flight and everything is waited for.
        if (issued - i >= S - 1) wait_vmcnt<(S - 2) * LPW>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();   // everyone's part of stage i is in LDS; compute(i-1) done
        if (ld.has) issue(fill);
        compute(buf);
        buf = buf + 1 == S ? 0 : buf + 1;
        fill = fill + 1 == S ? 0 : fill + 1;
    }

    // ---- a chunk of a split block row: park the tile; the last chunk to arrive adds them up ----
    // The tiles and the counter are accessed with device-scope atomic operations (relaxed), which
    // go to memory past the per-XCD L2: a tile stored on one XCD is read on another without
    // writing back or invalidating a whole L2, which device-scope fences would do.  Order: every
    // wavefront waits until its stores are acknowledged, the workgroup meets at a barrier, then
    // one lane counts the arrival; the workgroup that counts the last one reads all tiles.
    if (split >= 0) {
        constexpr int TILE_FLOATS = MI * NI * 16 * 64;  // per wavefront
        const int64_t tile_set = (int64_t)map.ntiles * WAVES * TILE_FLOATS;  // floats per chunk
        float* const mine = plan.partials + (int64_t)(first_part + chunk) * tile_set +
                            ((int64_t)tile * WAVES + wave) * TILE_FLOATS + lane;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    __hip_atomic_store(mine + ((mi * NI + ni) * 16 + r) * 64, acc[mi][ni][r], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();   // every wavefront's tile is in memory, and the ring is idle: its first
                           // word carries the verdict (a variable of its own would cost a workgroup per CU)
        volatile int32_t* const last_flag = reinterpret_cast<volatile int32_t*>(lds);
        if (tid == 0) {
            int32_t* const counter = plan.counters + (int64_t)split * map.ntiles + tile;
            const int32_t before = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *last_flag = before == nchunks - 1;
            if (before == nchunks - 1)   // ready for the next launch
                __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        const bool last_chunk = *last_flag != 0;
        __syncthreads();   // the flag is read before the ring is reused below
        if (!last_chunk) return;
        const float* const first = plan.partials + (int64_t)first_part * tile_set +
                                   ((int64_t)tile * WAVES + wave) * TILE_FLOATS + lane;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
        for (int32_t c = 0; c < nchunks; ++c) {   // fixed order: the sum does not depend on who came last
            const float* src = first + (int64_t)c * tile_set;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        acc[mi][ni][r] += __hip_atomic_load(src + ((mi * NI + ni) * 16 + r) * 64, __ATOMIC_RELAXED,
                                                            __HIP_MEMORY_SCOPE_AGENT);
        }
    }

    // ---- epilogue: acc holds the transposed tiles: lane -> output row lane%32 (+32*mi),
    // register quad q -> columns 32*ni + 8*q + 4*(lane/32) .. +3 of the wavefront's NI*32 columns
    TC* C = static_cast<TC*>(p.C);
    const bool accumulate = p.accumulate != 0;
    const int64_t wcol0 = ntile0 + NI * 32 * wave;
    if constexpr (sizeof(TC) == 2) {
        if (!accumulate) {
            // 16-bit C: round, park the wavefront's bM x (NI*32) tile in LDS (the ring is idle now)
            // and write it out as full row segments, 16 bytes per lane.
            constexpr int CSTRIDE = NI * 64 + 16;  // bytes per staged row (NI*64 of data)
            constexpr int LPR = NI * 4;            // lanes per row
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
            const int64_t col = wcol0 + 8 * (lane % LPR);
#pragma unroll
            for (int it = 0; it < BM / (64 / LPR); ++it) {
                const int r = it * (64 / LPR) + lane / LPR;
                const u32x4 v = *reinterpret_cast<const u32x4*>(cw + r * CSTRIDE + (lane % LPR) * 16);
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
                const int64_t col = wcol0 + 32 * ni + 8 * q + 4 * (lane / 32);
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

// ---- plan kernels -------------------------------------------------------------------------
// hist[b]: work items whose length class is b (class 0 = longest); misc: 0 split rows,
// 1 chunks of split rows, 2 and 3 the cursors that hand out split ids and partial tile sets.
struct PlanScratch {
    int32_t* hist;    // [kPlanBuckets]
    int32_t* start;   // [kPlanBuckets]
    int32_t* cursor;  // [kPlanBuckets]
    int32_t* misc;    // [4]
};

__global__ void k_plan_zero(PlanScratch sc) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < kPlanBuckets) {
        sc.hist[i] = 0;
        sc.cursor[i] = 0;
    }
    if (i < 4) sc.misc[i] = 0;
}

struct RowCut {
    int64_t p0, p1;
    int32_t nchunks, chunk_len, bucket;
};

__device__ inline RowCut cut_row(const int32_t* __restrict__ AM, int64_t G, int64_t r, int32_t chunk_groups) {
    RowCut c;
    c.p0 = lower_bound_i32(AM, G, (int32_t)r);
    c.p1 = lower_bound_i32(AM, G, (int32_t)r + 1);
    const int64_t len = c.p1 - c.p0;
    c.nchunks = len > chunk_groups ? (int32_t)ceil_div(len, chunk_groups) : 1;
    c.chunk_len = (int32_t)ceil_div(len, c.nchunks);
    c.bucket = kPlanBuckets - 1 - (c.chunk_len < kPlanBuckets - 1 ? c.chunk_len : kPlanBuckets - 1);
    return c;
}

__global__ void k_plan_count(const int32_t* __restrict__ AM, int64_t G, int64_t nrows, int32_t chunk_groups,
                             PlanScratch sc) {
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r >= nrows) return;
    const RowCut c = cut_row(AM, G, r, chunk_groups);
    atomicAdd(&sc.hist[c.bucket], c.nchunks);
    if (c.nchunks > 1) {
        atomicAdd(&sc.misc[0], 1);
        atomicAdd(&sc.misc[1], c.nchunks);
    }
}

// One workgroup of kPlanBuckets threads: exclusive prefix sums of the class counts, header.
__global__ void k_plan_scan(PlanScratch sc, PlanHeader* hdr, PlanHeader value) {
    __shared__ int32_t s[kPlanBuckets];
    const int t = threadIdx.x;
    const int32_t mine = sc.hist[t];
    s[t] = mine;
    __syncthreads();
    for (int d = 1; d < kPlanBuckets; d *= 2) {
        const int32_t v = t >= d ? s[t - d] : 0;
        __syncthreads();
        s[t] += v;
        __syncthreads();
    }
    sc.start[t] = s[t] - mine;
    if (t == kPlanBuckets - 1) {
        value.n_items = s[t];
        value.n_split_rows = sc.misc[0];
        value.n_chunks = sc.misc[1];
        *hdr = value;
    }
}

__global__ void k_plan_fill(const int32_t* __restrict__ AM, int64_t G, int64_t nrows, int32_t chunk_groups,
                            int32_t ntiles, PlanScratch sc, PlanItem* __restrict__ items,
                            int32_t* __restrict__ counters) {
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r >= nrows) return;
    const RowCut c = cut_row(AM, G, r, chunk_groups);
    PlanItem it;
    it.row = (int32_t)r;
    it.nchunks = c.nchunks;
    it.reserved = 0;
    if (c.nchunks == 1) {
        it.p0 = (int32_t)c.p0;
        it.p1 = (int32_t)c.p1;
        it.split = -1;
        it.chunk = 0;
        it.first_part = 0;
        items[sc.start[c.bucket] + atomicAdd(&sc.cursor[c.bucket], 1)] = it;
        return;
    }
    it.split = atomicAdd(&sc.misc[2], 1);
    it.first_part = atomicAdd(&sc.misc[3], c.nchunks);
    for (int32_t t = 0; t < ntiles; ++t) counters[(int64_t)it.split * ntiles + t] = 0;
    for (int32_t k = 0; k < c.nchunks; ++k) {
        const int64_t a = c.p0 + (int64_t)k * c.chunk_len, b = a + c.chunk_len;
        it.p0 = (int32_t)(a < c.p1 ? a : c.p1);
        it.p1 = (int32_t)(b < c.p1 ? b : c.p1);
        it.chunk = k;
        items[sc.start[c.bucket] + atomicAdd(&sc.cursor[c.bucket], 1)] = it;
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

// ---- tiling ---------------------------------------------------------------------------------
// Four wavefronts of 64 columns each, one stored block x 32 values of k per step, ring of four
// stages (80 KB of LDS for 64-row blocks: two workgroups per CU).  Measured alternatives on the
// two benchmark shapes, all slower: two steps per stage with a two- or three-stage ring
// (one barrier per 64 values of k), 128-column tiles with two wavefronts, 128-column tiles
// with four wavefronts of 32 columns.
constexpr int kWaves = 4, kNI = 2, kStages = 4;
constexpr int kNT = kWaves * kNI * 32;

int wg_per_cu(int32_t bM) { return std::max(1, (160 * 1024) / (kStages * (8 * (kNT / 128) + bM / 16) * 1024)); }

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

// Where the parts of a plan sit in the workspace; a function of the sizes only, so that the
// planning call and the SpMM call agree without reading anything back.
struct PlanLayout {
    int64_t chunk_groups, max_items, max_split_rows, max_chunks, ntiles;
    size_t off_scratch, off_items, off_counters, off_partials, total;
};

PlanLayout plan_layout(int64_t M, int64_t N, int64_t G, int32_t g, int32_t bM) {
    PlanLayout L;
    const int64_t nrows = M / bM;
    L.ntiles = std::max<int64_t>(1, ceil_div(N, kNT));
    // Workgroup slots of the chip that work on different block rows at a time.  A block row is
    // split when it holds more than twice the mean load of such a slot, and never below 64
    // slots: every chunk pays a workgroup's start-up and the round trip of its partial tile
    // (measured: splitting the moderately long rows of a uniform matrix loses more than the
    // shorter tail gains).
    const int64_t row_slots = std::max<int64_t>(1, 256LL * wg_per_cu(bM) / L.ntiles);
    const int64_t min_chunk = std::max<int64_t>(1, ceil_div(64, g));
    L.chunk_groups = std::min<int64_t>(1 << 30, std::max(min_chunk, ceil_div(2 * G, row_slots)));
    L.max_items = nrows + G / L.chunk_groups;
    L.max_split_rows = G / L.chunk_groups;
    L.max_chunks = 2 * (G / L.chunk_groups);
    size_t off = 256;  // header
    L.off_scratch = off;
    off += align_up((3 * kPlanBuckets + 4) * sizeof(int32_t), 256);
    L.off_items = off;
    off += align_up((size_t)std::max<int64_t>(L.max_items, 1) * sizeof(PlanItem), 256);
    L.off_counters = off;
    off += align_up((size_t)std::max<int64_t>(L.max_split_rows * L.ntiles, 1) * sizeof(int32_t), 256);
    L.off_partials = off;
    off += align_up((size_t)L.max_chunks * (size_t)L.ntiles * (size_t)bM * (size_t)kNT * sizeof(float), 256);
    L.total = off + 256;  // room to align the caller's pointer
    return L;
}

char* aligned_base(void* workspace) {
    return reinterpret_cast<char*>((reinterpret_cast<uintptr_t>(workspace) + 255) / 256 * 256);
}

bool mfma_shape(int64_t M, int64_t N, int32_t bM, int32_t bK) {
    return (bM == 32 || bM == 64 || bM == 128) && bK % 32 == 0 && N % 8 == 0 && N >= 8 &&
           (M / bM) * ceil_div(N, 128) < (1LL << 31) - 8;
}

template <typename T, typename TC, int BM>
void launch_mfma(const BlockParams& p, const PlanView& view, int64_t items, hipStream_t s) {
    int64_t grid = 0;
    const TileMap map = make_map(items, ceil_div(p.N, kNT), grid);
    hipLaunchKernelGGL((spmm_block_mfma<T, TC, BM, kWaves, kNI, kStages>), dim3((unsigned)grid),
                       dim3(kWaves * 64), 0, s, p, map, view);
}

template <typename T, typename TC>
void launch_typed(const BlockParams& p, bool mfma_ok, const PlanView& view, int64_t items, hipStream_t s) {
    if constexpr (sizeof(T) == 2) {
        if (mfma_ok && p.bM == 32) return launch_mfma<T, TC, 32>(p, view, items, s);
        if (mfma_ok && p.bM == 64) return launch_mfma<T, TC, 64>(p, view, items, s);
        if (mfma_ok && p.bM == 128) return launch_mfma<T, TC, 128>(p, view, items, s);
    }
    const dim3 grid((unsigned)(p.M / p.bM), (unsigned)ceil_div(p.N, 256));
    hipLaunchKernelGGL((spmm_block_general<T, TC>), grid, dim3(256), 0, s, p);
}

}  // namespace
}  // namespace insum

using namespace insum;

extern "C" size_t insum_spmm_blockgroupcoo_workspace_bytes(int64_t M, int64_t N, int64_t G, int32_t g,
                                                           int32_t bM, int32_t bK) {
    if (M <= 0 || N <= 0 || G <= 0 || g <= 0 || bM <= 0 || bK <= 0 || M % bM) return 0;
    if (M >= (1LL << 31) || N >= (1LL << 31) || G >= (1LL << 31)) return 0;   // beyond what the SpMM accepts
    if (!mfma_shape(M, N, bM, bK)) return 0;  // the general kernel takes no plan
    return plan_layout(M, N, G, g, bM).total;
}

extern "C" insum_status insum_spmm_blockgroupcoo_plan(int64_t M, int64_t K, int64_t N, int64_t G, int32_t g,
                                                      int32_t bM, int32_t bK, const int32_t* AM,
                                                      void* workspace, size_t workspace_bytes, void* stream) {
    if (M < 0 || K < 0 || N < 0 || G < 0 || g <= 0 || bM <= 0 || bK <= 0) return INSUM_ERR_INVALID_ARG;
    if (M >= (1LL << 31) || K >= (1LL << 31) || N >= (1LL << 31)) return INSUM_ERR_INVALID_ARG;
    if (M % bM || K % bK) return INSUM_ERR_UNSUPPORTED;
    const size_t need = insum_spmm_blockgroupcoo_workspace_bytes(M, N, G, g, bM, bK);
    if (need == 0) return INSUM_OK;  // nothing to plan for this shape
    if (!AM) return INSUM_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < need) return INSUM_ERR_CAPACITY;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const PlanLayout L = plan_layout(M, N, G, g, bM);
    char* base = aligned_base(workspace);
    PlanScratch sc;
    sc.hist = reinterpret_cast<int32_t*>(base + L.off_scratch);
    sc.start = sc.hist + kPlanBuckets;
    sc.cursor = sc.start + kPlanBuckets;
    sc.misc = sc.cursor + kPlanBuckets;
    PlanHeader value{};
    value.magic = kPlanMagic;
    value.G = G;
    value.nrows = M / bM;
    value.AM = AM;
    value.g = g;
    value.bM = bM;
    value.ntiles = (int32_t)L.ntiles;
    value.nt = kNT;
    value.chunk_groups = (int32_t)L.chunk_groups;
    const int64_t nrows = M / bM;
    const unsigned row_blocks = (unsigned)std::max<int64_t>(1, ceil_div(nrows, 256));
    hipLaunchKernelGGL(k_plan_zero, dim3(kPlanBuckets / 256), dim3(256), 0, s, sc);
    hipLaunchKernelGGL(k_plan_count, dim3(row_blocks), dim3(256), 0, s, AM, G, nrows, (int32_t)L.chunk_groups, sc);
    hipLaunchKernelGGL(k_plan_scan, dim3(1), dim3(kPlanBuckets), 0, s, sc, reinterpret_cast<PlanHeader*>(base), value);
    hipLaunchKernelGGL(k_plan_fill, dim3(row_blocks), dim3(256), 0, s, AM, G, nrows, (int32_t)L.chunk_groups,
                       (int32_t)L.ntiles, sc, reinterpret_cast<PlanItem*>(base + L.off_items),
                       reinterpret_cast<int32_t*>(base + L.off_counters));
    INSUM_HIP_TRY(hipGetLastError());
    return INSUM_OK;
}

extern "C" insum_status insum_spmm_blockgroupcoo(int64_t M, int64_t K, int64_t N, int64_t G,
                                                 int32_t g, int32_t bM, int32_t bK,
                                                 const int32_t* AM, const int32_t* AK,
                                                 const void* AV, insum_dtype a_dt, const void* B,
                                                 int64_t ldb, insum_dtype b_dt, void* C,
                                                 int64_t ldc, insum_dtype c_dt, int accumulate,
                                                 void* workspace, size_t workspace_bytes,
                                                 void* stream) {
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

    const bool mfma_ok = b_dt != INSUM_F32 && mfma_shape(M, N, bM, bK) && ldb % 8 == 0 && ldb < (1LL << 27) &&
                         ldc % (c_dt == INSUM_F32 ? 4 : 8) == 0 &&
                         (reinterpret_cast<uintptr_t>(C) % 16) == 0 &&
                         (reinterpret_cast<uintptr_t>(B) % 16) == 0 &&
                         (reinterpret_cast<uintptr_t>(AV) % 16) == 0;
    PlanView view{};
    int64_t items = M / bM;
    const size_t need = insum_spmm_blockgroupcoo_workspace_bytes(M, N, G, g, bM, bK);
    if (mfma_ok && workspace && need > 0 && workspace_bytes >= need) {
        // The workspace may hold a plan; the kernel checks its header and falls back to whole
        // block rows in index order when it does not match this call.
        const PlanLayout L = plan_layout(M, N, G, g, bM);
        char* base = aligned_base(workspace);
        view.hdr = reinterpret_cast<const PlanHeader*>(base);
        view.items = reinterpret_cast<const PlanItem*>(base + L.off_items);
        view.counters = reinterpret_cast<int32_t*>(base + L.off_counters);
        view.partials = reinterpret_cast<float*>(base + L.off_partials);
        view.chunk_groups = (int32_t)L.chunk_groups;
        items = L.max_items;
    }
    if (b_dt == INSUM_F32) launch_typed<float, float>(p, false, view, items, s);
    else if (b_dt == INSUM_F16 && c_dt == INSUM_F16) launch_typed<__half, __half>(p, mfma_ok, view, items, s);
    else if (b_dt == INSUM_F16) launch_typed<__half, float>(p, mfma_ok, view, items, s);
    else if (c_dt == INSUM_BF16) launch_typed<bf16_t, bf16_t>(p, mfma_ok, view, items, s);
    else launch_typed<bf16_t, float>(p, mfma_ok, view, items, s);
    INSUM_HIP_TRY(hipGetLastError());
    return INSUM_OK;
}
