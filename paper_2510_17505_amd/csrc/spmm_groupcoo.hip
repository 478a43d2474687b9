// SpMM over GroupCOO for gfx950:  C[AM[p], n] (+)= sum_q AV[p,q] * B[AK[p,q], n]
// (paper: Section 4.1 GroupCOO equation; loop nest of the "GroupCOO SpMM" listing in
// Section 6.5, which keeps the group's sum in a register and scatters once per group).
//
// Design (bandwidth-bound: every stored slot gathers one row of B)
//   * The group list is cut into `runs` of equal length.  Because groups have a fixed
//     number of slots, equal runs are equal work whatever the row-length distribution.
//   * A run is owned by a "sub-wave": SW consecutive lanes of a wavefront, where SW lanes
//     x 16 bytes cover one row of B (SW = 32 for N = 128 fp32 or N = 256 fp16).  A
//     wavefront therefore gathers 64/SW rows per load instruction, each lane moving 16
//     bytes, and no cross-lane reduction is needed for the products.
//   * The run's slots are read with coalesced loads (lane j takes slot base+j: column,
//     value and the row of its group) and handed to the other lanes with cross-lane
//     shuffles, so the format is streamed exactly once; the next batch of slots is
//     requested before the current one is processed.  B rows are fetched eight slots at a
//     time before the first product is formed (8 x 16 B per lane in flight), with the eight
//     column shuffles issued back to back.  Which slots start a new row is one ballot per
//     batch, so the inner loop tests a bit instead of shuffling and comparing row ids.
//   * Wide B (more than 64 lanes x 16 bytes per row) is cut into column tiles; the tile
//     index is the fastest-varying part of the workgroup id, so with 8 tiles each XCD keeps
//     to one 1/8 column slice of B in its L2.
//   * Scatter is a segment reduction: AM is non-decreasing, so the sub-wave keeps the row
//     sum in registers while the row does not change and stores it once.  Rows between
//     two stored rows have no groups; the sub-wave that sees the jump writes their zeros,
//     so C needs no separate clearing pass - except that of a long gap it only writes the
//     ragged ends: the aligned 64-row chunks that lie wholly inside a gap are cleared, all in
//     parallel, by extra workgroups at the front of the launch (a chunk is such a chunk exactly when
//     no group's row falls into it: one binary search).
//   * Rows cut by a run boundary: the piece at the head of a run and the piece at its
//     tail go to an fp32 workspace; a second, tiny kernel adds the pieces of each such row
//     in run order and writes the row once.  No floating-point atomics: results are
//     reproducible, and 16-bit outputs are rounded exactly once.
#include <algorithm>
#include <initializer_list>

#include "common.h"

namespace insum {
namespace {

struct GroupParams {
    int64_t M, N, G;
    int32_t g, g_shift;  // g_shift = log2(g) when g is a power of two, else -1
    const int32_t* AM;
    const int32_t* AK;
    const void* AV;
    const void* B;
    int64_t ldb;
    void* C;
    int64_t ldc;
    int32_t accumulate;
    int64_t runs, groups_per_run;
    float* partial;  // [runs][2][npad]: 0 = head piece, 1 = tail piece
    int64_t npad;
    int32_t col_tiles;  // column tiles of SW*E columns; the tile index is the fastest part of blockIdx.x
};

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ inline int64_t imin(int64_t a, int64_t b) { return a < b ? a : b; }

// Streaming (read-once) loads of format data.
__device__ inline float load_stream(const float* p) { return __builtin_nontemporal_load(p); }
__device__ inline float load_stream(const __half* p) {
    const uint16_t u = __builtin_nontemporal_load(reinterpret_cast<const uint16_t*>(p));
    return __half2float(__ushort_as_half(u));
}
__device__ inline float load_stream(const bf16_t* p) {
    const uint16_t u = __builtin_nontemporal_load(reinterpret_cast<const uint16_t*>(p));
    return __uint_as_float(((uint32_t)u) << 16);
}

// ---- 16-byte (or scalar) row pieces --------------------------------------------------
template <typename T, int E>
struct Piece;  // raw storage of E consecutive elements of type T

template <>
struct Piece<float, 4> {
    f32x4 v;
    __device__ void load(const float* p) { v = *reinterpret_cast<const f32x4*>(p); }
    __device__ void zero() { v = f32x4{0.f, 0.f, 0.f, 0.f}; }
    __device__ void fma_into(float a, float (&acc)[4]) const {
        acc[0] = fmaf(a, v.x, acc[0]);
        acc[1] = fmaf(a, v.y, acc[1]);
        acc[2] = fmaf(a, v.z, acc[2]);
        acc[3] = fmaf(a, v.w, acc[3]);
    }
};
template <>
struct Piece<__half, 8> {
    u32x4 v;
    __device__ void load(const __half* p) { v = *reinterpret_cast<const u32x4*>(p); }
    __device__ void zero() { v = u32x4{0, 0, 0, 0}; }
    __device__ void fma_into(float a, float (&acc)[8]) const {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const __half2 h = *reinterpret_cast<const __half2*>(&w[i]);
            const float2 f = __half22float2(h);
            acc[2 * i] = fmaf(a, f.x, acc[2 * i]);
            acc[2 * i + 1] = fmaf(a, f.y, acc[2 * i + 1]);
        }
    }
};
template <>
struct Piece<bf16_t, 8> {
    u32x4 v;
    __device__ void load(const bf16_t* p) { v = *reinterpret_cast<const u32x4*>(p); }
    __device__ void zero() { v = u32x4{0, 0, 0, 0}; }
    __device__ void fma_into(float a, float (&acc)[8]) const {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[2 * i] = fmaf(a, __uint_as_float(w[i] << 16), acc[2 * i]);
            acc[2 * i + 1] = fmaf(a, __uint_as_float(w[i] & 0xffff0000u), acc[2 * i + 1]);
        }
    }
};
template <typename T>
struct Piece<T, 1> {
    T v;
    __device__ void load(const T* p) { v = *p; }
    __device__ void zero() { v = from_float<T>(0.f); }
    __device__ void fma_into(float a, float (&acc)[1]) const { acc[0] = fmaf(a, to_float(v), acc[0]); }
};

// Write E fp32 sums to a row of C (converted to TC), optionally adding what is there.
template <typename TC, int E>
__device__ inline void store_c(TC* dst, const float (&acc)[E], bool add_old) {
    float out[E];
#pragma unroll
    for (int i = 0; i < E; ++i) out[i] = acc[i];
    if (add_old) {
#pragma unroll
        for (int i = 0; i < E; ++i) out[i] += to_float(dst[i]);
    }
    if constexpr (E == 1) {
        dst[0] = from_float<TC>(out[0]);
    } else if constexpr (sizeof(TC) == 4) {
#pragma unroll
        for (int i = 0; i < E; i += 4)
            __builtin_nontemporal_store(f32x4{out[i], out[i + 1], out[i + 2], out[i + 3]},
                                        reinterpret_cast<f32x4*>(dst + i));
    } else {
        static_assert(E == 8, "16-bit outputs use 8 elements per lane");
        union {
            TC h[8];
            u32x4 u;
        } pk;
#pragma unroll
        for (int i = 0; i < 8; ++i) pk.h[i] = from_float<TC>(out[i]);
        __builtin_nontemporal_store(pk.u, reinterpret_cast<u32x4*>(dst));
    }
}

template <int E>
__device__ inline void store_partial(float* dst, const float (&acc)[E]) {
#pragma unroll
    for (int i = 0; i < E; ++i) dst[i] = acc[i];
}

constexpr int kGapChunk = 64;  // rows; aligned chunks inside a gap of empty rows are cleared by workgroups of their own

template <typename TC, int E>
__device__ inline void zero_rows(TC* C, int64_t ldc, int64_t n0, int64_t first, int64_t last_excl) {
    float z[E];
#pragma unroll
    for (int i = 0; i < E; ++i) z[i] = 0.f;
    for (int64_t r = first; r < last_excl; ++r) store_c<TC, E>(C + r * ldc + n0, z, false);
}

// Rows [first, last_excl) have no groups.  Clears those of them that do not belong to an
// aligned chunk of kGapChunk rows lying wholly inside the gap (at most 2 * (kGapChunk - 1) rows).
template <typename TC, int E>
__device__ inline void zero_gap_ends(TC* C, int64_t ldc, int64_t n0, int64_t first, int64_t last_excl) {
    if (first >= last_excl) return;
    const int64_t up = (first + kGapChunk - 1) / kGapChunk * kGapChunk;
    const int64_t lo = up < last_excl ? up : last_excl;
    const int64_t down = last_excl / kGapChunk * kGapChunk;
    const int64_t hi = down > lo ? down : lo;
    zero_rows<TC, E>(C, ldc, n0, first, lo);
    zero_rows<TC, E>(C, ldc, n0, hi, last_excl);
}

__device__ inline int64_t group_of_slot(int64_t slot, int32_t g, int32_t g_shift) {
    return g_shift >= 0 ? (slot >> g_shift) : (slot / g);
}

__device__ inline int64_t first_group_at_or_after(const int32_t* __restrict__ AM, int64_t G, int64_t row) {
    int64_t lo = 0, hi = G;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (AM[mid] < row) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

// ---- chunks of empty rows ------------------------------------------------------------------------
// A workgroup looks at kGapChunksPerBlock aligned chunks of kGapChunk rows: one thread per chunk
// decides whether any group's row falls into it (binary search), then the whole workgroup
// clears the chunks found empty, 16 bytes per lane where the layout allows.  These workgroups
// travel at the front of the main launch.
constexpr int kGapChunksPerBlock = 16;

template <typename TC>
__device__ inline void clear_empty_chunks(const GroupParams& p, int64_t chunk0) {
    __shared__ int32_t empty[kGapChunksPerBlock];
    if (threadIdx.x < kGapChunksPerBlock) {
        const int64_t chunk = chunk0 + threadIdx.x;
        bool is_empty = false;
        if (chunk < p.M / kGapChunk) {
            const int64_t q = first_group_at_or_after(p.AM, p.G, chunk * kGapChunk);
            is_empty = q == p.G || p.AM[q] >= (chunk + 1) * kGapChunk;
        }
        empty[threadIdx.x] = is_empty;
    }
    __syncthreads();
    TC* const C = static_cast<TC*>(p.C);
    constexpr int V = 16 / (int)sizeof(TC);
    const bool vec = p.N % V == 0 && p.ldc % V == 0 && (reinterpret_cast<uintptr_t>(C) % 16) == 0;
    for (int c = 0; c < kGapChunksPerBlock; ++c) {
        if (!empty[c]) continue;   // the same decision in every thread
        TC* rows = C + (chunk0 + c) * kGapChunk * p.ldc;
        if (vec) {
            const int64_t per_row = p.N / V;
            for (int r = 0; r < kGapChunk; ++r)
                for (int64_t j = threadIdx.x; j < per_row; j += 256)
                    __builtin_nontemporal_store(u32x4{0, 0, 0, 0}, reinterpret_cast<u32x4*>(rows + r * p.ldc) + j);
        } else {
            for (int r = 0; r < kGapChunk; ++r)
                for (int64_t j = threadIdx.x; j < p.N; j += 256) rows[r * p.ldc + j] = from_float<TC>(0.f);
        }
    }
}

// ---- main kernel ---------------------------------------------------------------------
template <typename TB, typename TC, int E, int SW>
__global__ __launch_bounds__(256) void spmm_groupcoo_main(GroupParams p, unsigned gap_blocks) {
    constexpr int U = SW >= 8 ? 8 : SW;  // rows of B in flight per lane
    if (blockIdx.x < gap_blocks) return clear_empty_chunks<TC>(p, (int64_t)blockIdx.x * kGapChunksPerBlock);
    const unsigned block = blockIdx.x - gap_blocks;
    // Workgroup id = run block * col_tiles + column tile.  Consecutive ids go to different
    // XCDs, so with 8 (or 2, 4) column tiles every XCD keeps to its own columns of B and its
    // L2 holds a 1/8 slice instead of all of B.
    const int lane = threadIdx.x % SW;
    const int64_t run = ((int64_t)(block / p.col_tiles) * 256 + threadIdx.x) / SW;
    if (run >= p.runs) return;  // the SW lanes of a sub-wave leave together
    const int64_t n0 = ((int64_t)(block % p.col_tiles) * SW + lane) * E;
    const bool col_ok = n0 < p.N;

    const TB* __restrict__ B = static_cast<const TB*>(p.B);
    const TB* __restrict__ AV = static_cast<const TB*>(p.AV);
    const int32_t* __restrict__ AK = p.AK;
    const int32_t* __restrict__ AM = p.AM;
    TC* C = static_cast<TC*>(p.C);
    const bool accumulate = p.accumulate != 0;

    const int64_t gs = run * p.groups_per_run;
    const int64_t ge = imin(p.G, gs + p.groups_per_run);
    const int64_t slot_end = ge * p.g;
    const int32_t first_row = AM[gs];
    const int32_t prev_row = gs > 0 ? AM[gs - 1] : -1;
    const int32_t last_row = AM[ge - 1];
    const bool tail_cont = ge < p.G && AM[ge] == last_row;

    float acc[E];
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] = 0.f;
    int32_t cur = first_row;
    bool cur_is_head = prev_row == first_row;  // this row began in an earlier run
    float* const my_partial = p.partial + (run * 2) * p.npad + n0;

    if (!accumulate && !cur_is_head && col_ok) zero_gap_ends<TC, E>(C, p.ldc, n0, (int64_t)prev_row + 1, first_row);

    // Lanes beyond N (ragged last column tile) gather column 0 and never store.
    const TB* const Bcol = B + (col_ok ? n0 : 0);
    const int sub_base = (threadIdx.x % 64) / SW * SW;  // first lane of this sub-wave in the wavefront

    // One coalesced read of SW slots of the format: lane j gets slot sb+j.
    auto load_meta = [&](int64_t sb, int32_t& ak, float& av, int32_t& am) {
        const int64_t my = sb + lane;
        ak = 0;
        av = 0.f;
        am = -1;
        if (my < slot_end) {
            ak = __builtin_nontemporal_load(AK + my);
            av = load_stream(AV + my);
            am = AM[group_of_slot(my, p.g, p.g_shift)];
        }
    };
    // The row sum of `cur` is complete (inside this run): store it, zero-fill skipped rows.
    auto flush = [&](int32_t next_row) {
        if (col_ok) {
            if (cur_is_head) store_partial<E>(my_partial, acc);
            else store_c<TC, E>(C + (int64_t)cur * p.ldc + n0, acc, accumulate);
            if (!accumulate) zero_gap_ends<TC, E>(C, p.ldc, n0, (int64_t)cur + 1, next_row);
        }
        cur_is_head = false;
        cur = next_row;
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] = 0.f;
    };

    int32_t ak_l, am_l, ak_n = 0, am_n = -1;
    float av_l, av_n = 0.f;
    load_meta(gs * p.g, ak_l, av_l, am_l);
    for (int64_t sb = gs * p.g; sb < slot_end; sb += SW) {
        if (sb + SW < slot_end) load_meta(sb + SW, ak_n, av_n, am_n);  // next batch, in flight during this one
        const int nb = (int)imin((int64_t)SW, slot_end - sb);
        // Which slots start a new row: bit j of `starts` (identical in all lanes of the sub-wave).
        int32_t am_prev = __shfl_up(am_l, 1, SW);
        if (lane == 0) am_prev = cur;
        const uint64_t starts = (__ballot(lane < nb && am_l != am_prev) >> sub_base);
#pragma unroll
        for (int c = 0; c < SW; c += U) {
            if (c >= nb) break;
            Piece<TB, E> rowpiece[U];
            int32_t col[U];
#pragma unroll
            for (int u = 0; u < U; ++u) col[u] = __shfl(ak_l, c + u, SW);
#pragma unroll
            for (int u = 0; u < U; ++u)  // gather: U rows of B, 16 bytes per lane each
                rowpiece[u].load(Bcol + (int64_t)col[u] * p.ldb);
            float a[U];
#pragma unroll
            for (int u = 0; u < U; ++u) a[u] = __shfl(av_l, c + u, SW);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (c + u < nb) {  // slots past the end of the run hold column 0 and value 0
                    if ((starts >> (c + u)) & 1) flush(__shfl(am_l, c + u, SW));
                    rowpiece[u].fma_into(a[u], acc);
                }
            }
        }
        ak_l = ak_n;
        av_l = av_n;
        am_l = am_n;
    }
    if (col_ok) {
        if (cur_is_head) store_partial<E>(my_partial, acc);
        else if (tail_cont) store_partial<E>(my_partial + p.npad, acc);
        else store_c<TC, E>(C + (int64_t)cur * p.ldc + n0, acc, accumulate);
        if (ge == p.G && !accumulate) zero_gap_ends<TC, E>(C, p.ldc, n0, (int64_t)cur + 1, p.M);
    }
}

// ---- rows shared between runs ------------------------------------------------------------------
// Run r owns the row at its tail when that row starts inside r and continues into r+1.
// Its sum is tail(r) + head(r+1) + ... + head(last), where `last` is the run that holds the row's
// last group (for a long row found by binary search), so that the pieces are independent loads.
// A row of up to kLongSpan pieces is added up by the sub-wave of its run.  A longer one (a hub
// row) is added up by the whole workgroup: sub-wave j takes the pieces j, j + NSUB, ... and the
// NSUB sums are combined in sub-wave order through LDS - a fixed order either way.
constexpr int kLongSpan = 8;

// acc += head(k) for k = first, first + stride, ... <= last, four loads in flight
template <int E>
__device__ inline void add_heads(const float* __restrict__ partial, int64_t npad, int64_t n0, int64_t first,
                                 int64_t last, int64_t stride, float (&acc)[E]) {
    int64_t k = first;
    for (; k + 3 * stride <= last; k += 4 * stride) {
        float piece[4][E];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < E; ++i) piece[u][i] = partial[((k + u * stride) * 2) * npad + n0 + i];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < E; ++i) acc[i] += piece[u][i];
    }
    for (; k <= last; k += stride) {
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] += partial[(k * 2) * npad + n0 + i];
    }
}

template <typename TC, int E, int SW>
__global__ __launch_bounds__(256) void spmm_groupcoo_seams(GroupParams p) {
    constexpr int NSUB = 256 / SW;
    __shared__ int64_t long_run[NSUB], long_last[NSUB];   // hub rows owned by this workgroup's runs
    __shared__ int32_t long_row[NSUB];
    __shared__ float part[256 * E];
    const int lane = threadIdx.x % SW, sub = threadIdx.x / SW;
    const int64_t run = ((int64_t)(blockIdx.x / p.col_tiles) * 256 + threadIdx.x) / SW;
    const int64_t n0 = ((int64_t)(blockIdx.x % p.col_tiles) * SW + lane) * E;
    const bool col_ok = n0 < p.N;
    const int32_t* __restrict__ AM = p.AM;
    TC* const C = static_cast<TC*>(p.C);

    bool owner = false;
    int32_t row = 0;
    int64_t last = 0;
    if (run < p.runs) {
        const int64_t gs = run * p.groups_per_run;
        const int64_t ge = imin(p.G, gs + p.groups_per_run);
        row = AM[ge - 1];
        // the tail row goes on into the next run, and did not begin in an earlier one
        owner = ge < p.G && AM[ge] == row && !(gs > 0 && AM[gs - 1] == row);
        if (owner) {
            // Most shared rows end in the next run or two: look at the first group of the next
            // kLongSpan + 2 runs (independent loads), and search only when the row is still going on.
            int32_t begins[kLongSpan + 1];   // row at the start of run + 2 + k (-1 past the end)
#pragma unroll
            for (int k = 0; k <= kLongSpan; ++k) {
                const int64_t ke = (run + 2 + k) * p.groups_per_run;
                begins[k] = ke < p.G ? AM[ke] : -1;
            }
            bool ended = false;
            last = run + kLongSpan + 2;
#pragma unroll
            for (int k = kLongSpan; k >= 0; --k) {
                if (begins[k] != row) {
                    ended = true;
                    last = run + 1 + k;
                }
            }
            if (!ended) last = (first_group_at_or_after(AM, p.G, (int64_t)row + 1) - 1) / p.groups_per_run;
        }
    }
    const bool is_long = owner && last - run > kLongSpan;
    if (lane == 0) {
        long_run[sub] = is_long ? run : -1;
        long_last[sub] = last;
        long_row[sub] = row;
    }
    if (owner && !is_long && col_ok) {
        float acc[E];
        const float* tail = p.partial + (run * 2 + 1) * p.npad + n0;
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] = tail[i];
        add_heads<E>(p.partial, p.npad, n0, run + 1, last, 1, acc);
        store_c<TC, E>(C + (int64_t)row * p.ldc + n0, acc, p.accumulate != 0);
    }
    __syncthreads();
    for (int s = 0; s < NSUB; ++s) {
        const int64_t r = long_run[s];   // the same in every thread
        if (r < 0) continue;
        float acc[E];
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] = 0.f;
        if (col_ok) add_heads<E>(p.partial, p.npad, n0, r + 1 + sub, long_last[s], NSUB, acc);
#pragma unroll
        for (int i = 0; i < E; ++i) part[(sub * SW + lane) * E + i] = acc[i];
        __syncthreads();
        if (sub == 0 && col_ok) {
            const float* tail = p.partial + (r * 2 + 1) * p.npad + n0;
#pragma unroll
            for (int i = 0; i < E; ++i) acc[i] = tail[i];
            for (int j = 0; j < NSUB; ++j)
#pragma unroll
                for (int i = 0; i < E; ++i) acc[i] += part[(j * SW + lane) * E + i];
            store_c<TC, E>(C + (int64_t)long_row[s] * p.ldc + n0, acc, p.accumulate != 0);
        }
        __syncthreads();
    }
}

template <typename TC>
__global__ __launch_bounds__(256) void fill_zero_2d(TC* C, int64_t ldc, int64_t M, int64_t N) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= M * N) return;
    C[(i / N) * ldc + (i % N)] = static_cast<TC>(0);
}

// ---- launch planning -----------------------------------------------------------------
struct Plan {
    int E, SW;
    int64_t col_tiles, groups_per_run, runs;
};

int next_pow2(int64_t x) {   // smallest power of two >= x, at most 2^30
    int p = 1;
    while (p < x && p < (1 << 30)) p <<= 1;
    return p;
}

// elem_size: bytes per element of B; vec: 16-byte path usable.
// run_cap > 0 limits the number of runs (a caller with a fixed amount of scratch).
Plan make_plan(int64_t N, int64_t G, int32_t g, int elem_size, bool vec, int64_t run_cap = 0) {
    Plan pl;
    pl.E = vec ? 16 / elem_size : 1;
    const int64_t chunks = ceil_div(N, pl.E);
    if (vec) {
        pl.SW = (int)std::min<int64_t>(64, std::max<int64_t>(4, next_pow2(chunks)));
    } else {
        pl.SW = chunks <= 16 ? 16 : 64;
    }
    pl.col_tiles = ceil_div(chunks, pl.SW);
    // At most two runs per sub-wave slot of the chip (256 CUs x 32 wavefronts), never fewer than
    // two SW-slot batches per run.  A run also costs a start-up (its rows' bounds from AM, the
    // first batch of slots) and two partial rows for the seam pass, which weigh on runs of a few
    // batches: runs grow towards 256 slots as long as half of the chip's sub-wave slots still get
    // one (cfg2: 64 -> 224 slots per run, 63 -> 56 us; the large workloads are unaffected).
    const int64_t subwaves = 256LL * 32 * (64 / pl.SW);
    int64_t target_runs = std::max<int64_t>(1, 2 * subwaves / pl.col_tiles);
    if (run_cap > 0) target_runs = std::min(target_runs, run_cap);
    const int64_t min_groups = std::max<int64_t>(1, ceil_div(2 * pl.SW, g));
    int64_t gpr = std::max<int64_t>(min_groups, ceil_div(G, target_runs));
    const int64_t preferred = std::max<int64_t>(min_groups, ceil_div(256, g));
    if (gpr < preferred) {
        const int64_t half_chip = std::max<int64_t>(1, subwaves / 2 / pl.col_tiles);
        gpr = std::min(preferred, std::max(gpr, ceil_div(G, half_chip)));
    }
    pl.groups_per_run = gpr;
    pl.runs = G > 0 ? ceil_div(G, pl.groups_per_run) : 0;
    return pl;
}

int64_t padded_cols(int64_t N) { return (N + 7) / 8 * 8; }

template <typename TB, typename TC, int E, int SW>
void launch_pair(const GroupParams& p, const Plan& pl, hipStream_t s) {
    const unsigned seam_blocks = (unsigned)(ceil_div(p.runs, 256 / SW) * pl.col_tiles);
    // nothing to clear when C is accumulated into
    const unsigned gap_blocks = p.accumulate ? 0u : (unsigned)ceil_div(p.M / kGapChunk, kGapChunksPerBlock);
    hipLaunchKernelGGL((spmm_groupcoo_main<TB, TC, E, SW>), dim3(gap_blocks + seam_blocks), dim3(256), 0, s, p,
                       gap_blocks);
    hipLaunchKernelGGL((spmm_groupcoo_seams<TC, E, SW>), dim3(seam_blocks), dim3(256), 0, s, p);
}

template <typename TB, typename TC>
void launch_typed(const GroupParams& p, const Plan& pl, hipStream_t s) {
    constexpr int EV = 16 / (int)sizeof(TB);
    if (pl.E == 1) {
        if (pl.SW == 16) launch_pair<TB, TC, 1, 16>(p, pl, s);
        else launch_pair<TB, TC, 1, 64>(p, pl, s);
        return;
    }
    switch (pl.SW) {
        case 4: launch_pair<TB, TC, EV, 4>(p, pl, s); break;
        case 8: launch_pair<TB, TC, EV, 8>(p, pl, s); break;
        case 16: launch_pair<TB, TC, EV, 16>(p, pl, s); break;
        case 32: launch_pair<TB, TC, EV, 32>(p, pl, s); break;
        default: launch_pair<TB, TC, EV, 64>(p, pl, s); break;
    }
}

}  // namespace
}  // namespace insum

using namespace insum;

extern "C" size_t insum_spmm_groupcoo_workspace_bytes(int64_t M, int64_t N, int64_t G, int32_t g) {
    (void)M;
    if (N <= 0 || G <= 0 || g <= 0) return 256;
    if (N >= (1LL << 31) || G >= (1LL << 40)) return 0;   // beyond what the SpMM accepts
    int64_t runs = 0;
    for (int es : {2, 4})
        for (bool vec : {false, true}) runs = std::max(runs, make_plan(N, G, g, es, vec).runs);
    return align_up((size_t)runs * 2 * (size_t)padded_cols(N) * sizeof(float), 256) + 256;
}

namespace insum {
namespace {

// Shared body of the two entry points.  `scratch` is 256-byte aligned device memory of
// `scratch_bytes` bytes for the seam partials; run_cap as in make_plan.
insum_status spmm_groupcoo_run(int64_t M, int64_t K, int64_t N, int64_t G, int32_t g,
                               const int32_t* AM, const int32_t* AK, const void* AV, insum_dtype a_dt,
                               const void* B, int64_t ldb, insum_dtype b_dt, void* C, int64_t ldc,
                               insum_dtype c_dt, int accumulate, float* scratch, size_t scratch_bytes,
                               int64_t run_cap, hipStream_t s) {
    if (G == 0) {
        if (!accumulate) {
            if (ceil_div(M * N, 256) >= (1LL << 31)) return INSUM_ERR_UNSUPPORTED;
            const unsigned blocks = (unsigned)ceil_div(M * N, 256);
            if (c_dt == INSUM_F32) hipLaunchKernelGGL(fill_zero_2d<float>, dim3(blocks), dim3(256), 0, s, (float*)C, ldc, M, N);
            else hipLaunchKernelGGL(fill_zero_2d<uint16_t>, dim3(blocks), dim3(256), 0, s, (uint16_t*)C, ldc, M, N);
            INSUM_HIP_TRY(hipGetLastError());
        }
        return INSUM_OK;
    }

    const int es = dtype_size(b_dt);
    const int ev = 16 / es;
    const bool vec = N % ev == 0 && ldb % ev == 0 && ldc % ev == 0 &&
                     (reinterpret_cast<uintptr_t>(B) % 16) == 0 &&
                     (reinterpret_cast<uintptr_t>(C) % 16) == 0;
    const Plan pl = make_plan(N, G, g, es, vec, run_cap);

    GroupParams p;
    p.M = M; p.N = N; p.G = G; p.g = g;
    p.g_shift = (g & (g - 1)) == 0 ? __builtin_ctz((unsigned)g) : -1;
    p.AM = AM; p.AK = AK; p.AV = AV; p.B = B; p.ldb = ldb; p.C = C; p.ldc = ldc;
    p.accumulate = accumulate ? 1 : 0;
    p.runs = pl.runs; p.groups_per_run = pl.groups_per_run;
    p.npad = padded_cols(N);
    p.col_tiles = (int32_t)pl.col_tiles;
    if (ceil_div(pl.runs, 256 / pl.SW) * pl.col_tiles >= (1LL << 31)) return INSUM_ERR_UNSUPPORTED;
    const size_t need = (size_t)pl.runs * 2 * (size_t)p.npad * sizeof(float);
    if (!scratch || need > scratch_bytes) return INSUM_ERR_CAPACITY;
    p.partial = scratch;

    if (b_dt == INSUM_F32) launch_typed<float, float>(p, pl, s);
    else if (b_dt == INSUM_F16 && c_dt == INSUM_F16) launch_typed<__half, __half>(p, pl, s);
    else if (b_dt == INSUM_F16) launch_typed<__half, float>(p, pl, s);
    else if (c_dt == INSUM_BF16) launch_typed<bf16_t, bf16_t>(p, pl, s);
    else launch_typed<bf16_t, float>(p, pl, s);
    INSUM_HIP_TRY(hipGetLastError());
    return INSUM_OK;
}

insum_status check_spmm_groupcoo_args(int64_t M, int64_t K, int64_t N, int64_t G, int32_t g,
                                      const int32_t* AM, const int32_t* AK, const void* AV, insum_dtype a_dt,
                                      const void* B, int64_t ldb, insum_dtype b_dt, void* C, int64_t ldc,
                                      insum_dtype c_dt, bool& nothing_to_do) {
    nothing_to_do = false;
    if (M < 0 || K < 0 || N < 0 || G < 0 || g <= 0) return INSUM_ERR_INVALID_ARG;
    if (M >= (1LL << 31) || K >= (1LL << 31) || N >= (1LL << 31) || G >= (1LL << 40)) return INSUM_ERR_INVALID_ARG;
    if (!dtype_valid(a_dt) || !dtype_valid(b_dt) || !dtype_valid(c_dt)) return INSUM_ERR_INVALID_ARG;
    if (a_dt != b_dt || (c_dt != b_dt && c_dt != INSUM_F32)) return INSUM_ERR_UNSUPPORTED;
    if (ldb < N || ldc < N) return INSUM_ERR_INVALID_ARG;
    if (M == 0 || N == 0) {
        nothing_to_do = true;
        return INSUM_OK;
    }
    if (!C) return INSUM_ERR_INVALID_ARG;
    if (G > 0 && (!AM || !AK || !AV || !B || K == 0)) return INSUM_ERR_INVALID_ARG;
    return INSUM_OK;
}

}  // namespace
}  // namespace insum

extern "C" insum_status insum_spmm_groupcoo(int64_t M, int64_t K, int64_t N, int64_t G, int32_t g,
                                            const int32_t* AM, const int32_t* AK, const void* AV,
                                            insum_dtype a_dt, const void* B, int64_t ldb,
                                            insum_dtype b_dt, void* C, int64_t ldc,
                                            insum_dtype c_dt, int accumulate, void* workspace,
                                            size_t workspace_bytes, void* stream) {
    bool done = false;
    const insum_status st = check_spmm_groupcoo_args(M, K, N, G, g, AM, AK, AV, a_dt, B, ldb, b_dt, C, ldc, c_dt, done);
    if (st != INSUM_OK || done) return st;
    const uintptr_t base = reinterpret_cast<uintptr_t>(workspace);
    const uintptr_t ws = (base + 255) / 256 * 256;
    if (G > 0 && (!workspace || ws > base + workspace_bytes)) return INSUM_ERR_CAPACITY;
    return spmm_groupcoo_run(M, K, N, G, g, AM, AK, AV, a_dt, B, ldb, b_dt, C, ldc, c_dt, accumulate,
                             reinterpret_cast<float*>(ws), workspace ? base + workspace_bytes - ws : 0, 0,
                             static_cast<hipStream_t>(stream));
}

// ---- entry point that allocates nothing ------------------------------------------------------
// For callers that cannot allocate device memory (code under HIP graph capture, tight serving
// loops): the seam partials live in a file-scope device array instead of a caller workspace.
// Every GPU the library runs on holds its own copy of the array until the process ends.
namespace insum {
namespace {

constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch`, per device; null until looked up

// The array's name is only a host-side handle; its device address comes from the runtime, once
// per device and with that device current.  Concurrent first calls may both look it up: they
// obtain the same address.
insum_status static_scratch(void** out) {
    int dev = -1;
    INSUM_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return INSUM_ERR_UNSUPPORTED;
    void* ptr = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!ptr) {
        INSUM_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return INSUM_ERR_HIP;
        __atomic_store_n(&g_scratch_ptr[dev], ptr, __ATOMIC_RELEASE);
    }
    *out = ptr;
    return INSUM_OK;
}

}  // namespace
}  // namespace insum

extern "C" insum_status insum_spmm_groupcoo_noalloc(int64_t M, int64_t K, int64_t N, int64_t G, int32_t g,
                                                    const int32_t* AM, const int32_t* AK, const void* AV,
                                                    insum_dtype a_dt, const void* B, int64_t ldb,
                                                    insum_dtype b_dt, void* C, int64_t ldc,
                                                    insum_dtype c_dt, int accumulate, void* stream) {
    bool done = false;
    insum_status st = check_spmm_groupcoo_args(M, K, N, G, g, AM, AK, AV, a_dt, B, ldb, b_dt, C, ldc, c_dt, done);
    if (st != INSUM_OK || done) return st;
    // Each run stores a head piece and a tail piece of padded_cols(N) floats; a run is the least
    // that can be scheduled, so a row of partials wider than the array cannot be served.
    const size_t per_run = 2 * (size_t)padded_cols(N) * sizeof(float);
    if (per_run > kStaticScratchBytes) return INSUM_ERR_CAPACITY;
    void* ptr = nullptr;
    st = static_scratch(&ptr);
    if (st != INSUM_OK) return st;
    // Every partial that the second kernel reads is written by the first kernel of the same
    // call, so what an earlier call left in the array never has to be cleared.
    return spmm_groupcoo_run(M, K, N, G, g, AM, AK, AV, a_dt, B, ldb, b_dt, C, ldc, c_dt, accumulate,
                             static_cast<float*>(ptr), kStaticScratchBytes,
                             (int64_t)(kStaticScratchBytes / per_run), static_cast<hipStream_t>(stream));
}
