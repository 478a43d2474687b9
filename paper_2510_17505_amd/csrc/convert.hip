// COO -> GroupCOO and COO -> BlockGroupCOO on the device (paper: Section 4.1).
//
// The paper fixes the result (fixed-length groups along rows / block rows, the row stored
// once per group, padding inside a row's last group) but not an algorithm.  Here:
//   1. one pass validates coordinates and forms a 64-bit sort key
//      (GroupCOO: row*K + col; blocks: ((block row, block col), position inside block));
//   2. a stable radix sort of (key, value bits) gives the canonical order (row, col, input
//      position): equal keys keep their input order, so the position never has to be stored,
//      and the values arrive already permuted (no random gather afterwards);
//   3. row (block-row) boundaries are read off the sorted keys, prefix sums of ceil(occ/g)
//      give each row's first group, and G goes back to the host;
//   4. one streaming pass writes every sorted entry to group = first_group[row] + rank/g,
//      slot = rank % g; the last entry of a row also writes that group's padding.
// Count mode (no output buffers) only needs per-row counts and uses an atomic histogram
// instead of the sort.  Values are moved as raw bits; there is no floating-point arithmetic,
// so the output is a pure function of the input.
//
// The kernel map of a sparse convolution (Section 6.4) is grouped along its offset z the same
// way: key = z*X + x, the sort carries (y, value bits) packed in 64 bits, and the offsets play
// the part of the rows.
//
// The GroupCOO of the transposed matrix (insum_groupcoo_transpose) reuses all of this: the slots
// that hold entries are numbered with a prefix sum and written out as COO with row and column
// exchanged, and the conversion above groups them.
//
// The device-wide stable radix sort and the prefix sums are in sort_scan.h; keys are 32 bits
// wide when the largest possible key fits (it does for every block workload here) and 64 bits
// otherwise, and only the digits such a key can have are sorted.
#include <cstring>

#include <algorithm>

#include "common.h"
#include "sort_scan.h"

namespace insum {
namespace {

constexpr int kThreads = 256;

inline unsigned blocks_for(int64_t n) { return (unsigned)std::max<int64_t>(1, ceil_div(n, kThreads)); }

int bits_for(uint64_t max_value) {  // number of low bits that can be set in [0, max_value]
    int b = 0;
    while (b < 64 && (max_value >> b) != 0) ++b;
    return std::max(b, 1);
}

// Division of sort keys by a per-launch constant (K, or bM*bK): a shift when it is a power
// of two, a 64-bit division otherwise.
struct Divisor {
    uint64_t d;
    int32_t shift;  // log2(d) or -1
    explicit Divisor(uint64_t v) : d(v), shift((v & (v - 1)) == 0 ? __builtin_ctzll(v) : -1) {}
    __device__ uint64_t div(uint64_t x) const { return shift >= 0 ? (x >> shift) : (x / d); }
    // 32-bit keys: same quotient with 32-bit arithmetic (d fits whenever the key does)
    __device__ uint32_t div(uint32_t x) const { return shift >= 0 ? (x >> shift) : (x / (uint32_t)d); }
};

// ---- workspace carving -------------------------------------------------------------------
struct Carver {
    uintptr_t cur, end;
    bool ok = true;
    Carver(void* base, size_t bytes) {
        cur = (reinterpret_cast<uintptr_t>(base) + 255) / 256 * 256;
        end = reinterpret_cast<uintptr_t>(base) + bytes;
        if (!base || cur > end) ok = false;
    }
    template <typename T>
    T* take(size_t count) {
        const size_t bytes = align_up(std::max<size_t>(count, 1) * sizeof(T), 256);
        if (!ok || cur + bytes > end) {
            ok = false;
            return nullptr;
        }
        T* p = reinterpret_cast<T*>(cur);
        cur += bytes;
        return p;
    }
};

struct Flags {  // device-side status words, copied to the host with the counts
    int32_t out_of_range;
    int32_t duplicate;
    int32_t total_a;  // GroupCOO: G.  Blocks: number of nonzero blocks
    int32_t total_b;  // Blocks: G
};

// ---- kernels shared by both formats -----------------------------------------------------------
__global__ void k_zero_i32(int32_t* p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) p[i] = 0;
}

// start[r] = index of the first sorted entry whose row (key / per_row) is >= r, for r in
// [0, nrows]; start[nrows] = nnz.  Thread i owns the rows in (row(i-1), row(i)].
template <typename KeyT>
__global__ void k_row_bounds(int64_t nnz, int64_t nrows, Divisor per_row,
                             const KeyT* __restrict__ key, int32_t* __restrict__ start) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i > nnz) return;
    const int64_t cur = i < nnz ? (int64_t)per_row.div(key[i]) : nrows;
    const int64_t prev = i > 0 ? (int64_t)per_row.div(key[i - 1]) : -1;
    for (int64_t r = prev + 1; r <= cur; ++r) start[r] = (int32_t)i;
}

// gpr[i] = ceil((start[i+1] - start[i]) / g) for i < n, gpr[n] = 0 (so that an exclusive
// scan over n+1 elements ends with the total)
__global__ void k_groups_from_bounds(int64_t n, const int32_t* __restrict__ start, int32_t g,
                                     int32_t* __restrict__ gpr) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i > n) return;
    gpr[i] = i < n ? (start[i + 1] - start[i] + g - 1) / g : 0;
}

// the same from per-row counts; in place
__global__ void k_groups_from_counts(int64_t n, int32_t* occ, int32_t g) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i > n) return;
    occ[i] = i < n ? (occ[i] + g - 1) / g : 0;
}

__global__ void k_store_total(const int32_t* src, int32_t* dst) { *dst = *src; }

template <typename V>
__global__ void k_fill_zero(V* p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) p[i] = (V)0;
}

// ---- kernels: GroupCOO ---------------------------------------------------------------------
template <typename KeyT, bool HISTOGRAM>
__global__ void k_group_keys(int64_t M, int64_t K, int64_t nnz, const int32_t* __restrict__ row,
                             const int32_t* __restrict__ col, KeyT* __restrict__ key,
                             int32_t* __restrict__ occ, Flags* flags) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= nnz) return;
    const int32_t r = row[i], c = col[i];
    const bool ok = r >= 0 && r < M && c >= 0 && c < K;
    if (!ok) flags->out_of_range = 1;
    if constexpr (HISTOGRAM) {
        if (ok) atomicAdd(&occ[r], 1);
    } else {
        key[i] = ok ? (KeyT)((uint64_t)r * (uint64_t)K + (uint64_t)c) : (KeyT)0;
    }
}

template <typename KeyT, typename V>
__global__ void k_group_fill(Divisor per_row, int64_t nnz, int32_t g, const KeyT* __restrict__ key,
                             const V* __restrict__ val, const int32_t* __restrict__ row_start,
                             const int32_t* __restrict__ grp_start, int32_t* __restrict__ AM,
                             int32_t* __restrict__ AK, V* __restrict__ AV) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= nnz) return;
    const KeyT k = key[i];
    const int64_t r = (int64_t)per_row.div(k);
    const int32_t c = (int32_t)((uint64_t)k - (uint64_t)r * per_row.d);
    const int32_t first = row_start[r];
    const int32_t rank = (int32_t)(i - first);
    const int32_t occ = row_start[r + 1] - first;
    const int64_t grp = (int64_t)grp_start[r] + rank / g;
    const int32_t slot = rank % g;
    const int64_t dst = grp * g + slot;
    AK[dst] = c;
    AV[dst] = val[i];
    if (slot == 0) AM[grp] = (int32_t)r;
    if (rank == occ - 1) {  // last entry of its row: pad the rest of the group
        for (int32_t q = slot + 1; q < g; ++q) {
            AK[grp * g + q] = c;
            AV[grp * g + q] = (V)0;
        }
    }
}

// ---- kernels: GroupCOO -> COO of the transposed matrix ------------------------------------------
// A slot holds an entry unless it is padding: value bits all zero and the column of the slot to
// its left (same group) repeated - the pattern the conversion above writes.
template <typename V>
__device__ inline bool slot_is_real(const int32_t* __restrict__ AK, const V* __restrict__ AV, int64_t i, int32_t g) {
    return i % g == 0 || AV[i] != (V)0 || AK[i] != AK[i - 1];
}

// real[i] = 1 for a slot with an entry, for i < slots; real[slots] = 0 (the scan's total)
template <typename V>
__global__ void k_real_slots(int64_t slots, int32_t g, const int32_t* __restrict__ AK, const V* __restrict__ AV,
                             int32_t* __restrict__ real) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i > slots) return;
    real[i] = i < slots && slot_is_real(AK, AV, i, g) ? 1 : 0;
}

// entry number offs[i] of the transposed matrix: (row, col, value) = (AK[i], AM[i / g], AV[i])
template <typename V>
__global__ void k_transposed_entries(int64_t slots, int32_t g, const int32_t* __restrict__ AM,
                                     const int32_t* __restrict__ AK, const V* __restrict__ AV,
                                     const int32_t* __restrict__ offs, int32_t* __restrict__ row,
                                     int32_t* __restrict__ col, V* __restrict__ val) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= slots || !slot_is_real(AK, AV, i, g)) return;
    const int32_t e = offs[i];
    row[e] = AK[i];
    col[e] = AM[i / g];
    val[e] = AV[i];
}

// ---- kernels: BlockGroupCOO ----------------------------------------------------------------
template <typename KeyT>
__global__ void k_block_keys(int64_t M, int64_t K, int64_t nnz, int32_t bM, int32_t bK,
                             const int32_t* __restrict__ row, const int32_t* __restrict__ col,
                             KeyT* __restrict__ key, Flags* flags) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= nnz) return;
    const int32_t r = row[i], c = col[i];
    if (r < 0 || r >= M || c < 0 || c >= K) {
        flags->out_of_range = 1;
        key[i] = 0;
        return;
    }
    const uint64_t nbc = (uint64_t)(K / bK);
    const uint64_t blk = (uint64_t)(r / bM) * nbc + (uint64_t)(c / bK);
    key[i] = (KeyT)((blk * (uint64_t)bM + (uint64_t)(r % bM)) * (uint64_t)bK + (uint64_t)(c % bK));
}

// On sorted keys: head[i] = 1 when entry i is the first of its block; counts blocks per
// block row; equal neighbouring keys are duplicate coordinates.  head has nnz+1 entries
// (the last is 0) so its exclusive scan ends with the number of blocks.
template <typename KeyT>
__global__ void k_block_heads(int64_t nnz, Divisor per_block, Divisor blocks_per_row,
                              const KeyT* __restrict__ key, int32_t* __restrict__ head,
                              int32_t* __restrict__ occ, Flags* flags) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i > nnz) return;
    if (i == nnz) {
        head[i] = 0;
        return;
    }
    const uint64_t blk = per_block.div(key[i]);
    int32_t h = 1;
    if (i > 0) {
        const KeyT prev = key[i - 1];
        if (prev == key[i]) flags->duplicate = 1;
        h = per_block.div(prev) != blk;
    }
    head[i] = h;
    if (h) atomicAdd(&occ[blocks_per_row.div(blk)], 1);
}

template <typename KeyT, typename V>
__global__ void k_block_fill(Divisor per_block, Divisor blocks_per_row, int64_t nnz, int32_t g,
                             const KeyT* __restrict__ key, const V* __restrict__ val,
                             const int32_t* __restrict__ head, const int32_t* __restrict__ blk_ord,
                             const int32_t* __restrict__ brow_start,
                             const int32_t* __restrict__ grp_start, int32_t* __restrict__ AM,
                             int32_t* __restrict__ AK, V* __restrict__ AV) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= nnz) return;
    const uint64_t k = key[i];
    const uint64_t blk = per_block.div(k);
    const uint64_t inside = k - blk * per_block.d;  // bm * bK + bk
    const int64_t br = (int64_t)blocks_per_row.div(blk);
    const int32_t bc = (int32_t)(blk - (uint64_t)br * blocks_per_row.d);
    // blk_ord is the exclusive scan of head: for a head entry it is the block's ordinal,
    // for the other entries of the block it is ordinal + 1.
    const int32_t is_head = head[i];
    const int32_t ord = blk_ord[i] - (is_head ? 0 : 1);
    const int32_t rank = ord - brow_start[br];
    const int32_t occ = brow_start[br + 1] - brow_start[br];
    const int64_t grp = (int64_t)grp_start[br] + rank / g;
    const int32_t slot = rank % g;
    AV[((grp * g + slot) * (int64_t)per_block.d) + (int64_t)inside] = val[i];
    if (is_head) {
        AK[grp * g + slot] = bc;
        if (slot == 0) AM[grp] = (int32_t)br;
        if (rank == occ - 1)
            for (int32_t q = slot + 1; q < g; ++q) AK[grp * g + q] = bc;
    }
}

// ---- kernels: kernel map grouped along z -------------------------------------------------------
constexpr int kLdsBins = 4096;  // offsets counted in LDS when Z is at most this

// Validates the coordinates.  Fill mode forms key = z*X + x and payload = (y << 32) | value
// bits.  Count mode adds to occ[z]: per work-group in LDS first when Z <= kLdsBins (a stencil
// has few offsets, so global atomics would all hit the same few words).
template <typename KeyT, typename V, bool HISTOGRAM>
__global__ void k_map_keys(int64_t X, int64_t Y, int64_t Z, int64_t nnz, const int32_t* __restrict__ mx,
                           const int32_t* __restrict__ my, const int32_t* __restrict__ mz,
                           const V* __restrict__ mv, KeyT* __restrict__ key,
                           uint64_t* __restrict__ payload, int32_t* __restrict__ occ, Flags* flags) {
    __shared__ int32_t bins[HISTOGRAM ? kLdsBins : 1];
    const bool lds = HISTOGRAM && Z <= kLdsBins;
    if constexpr (HISTOGRAM) {
        if (lds) {
            for (int b = threadIdx.x; b < Z; b += kThreads) bins[b] = 0;
            __syncthreads();
        }
    }
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < nnz) {
        const int32_t x = mx[i], y = my[i], z = mz[i];
        const bool ok = x >= 0 && x < X && y >= 0 && y < Y && z >= 0 && z < Z;
        if (!ok) flags->out_of_range = 1;
        if constexpr (HISTOGRAM) {
            if (ok) atomicAdd(lds ? &bins[z] : &occ[z], 1);
        } else {
            key[i] = ok ? (KeyT)((uint64_t)z * (uint64_t)X + (uint64_t)x) : (KeyT)0;
            payload[i] = ((uint64_t)(uint32_t)y << 32) | (uint64_t)mv[i];
        }
    }
    if constexpr (HISTOGRAM) {
        if (lds) {
            __syncthreads();
            for (int b = threadIdx.x; b < Z; b += kThreads)
                if (bins[b]) atomicAdd(&occ[b], bins[b]);
        }
    }
}

template <typename KeyT, typename V>
__global__ void k_map_fill(Divisor per_z, int64_t nnz, int32_t g, const KeyT* __restrict__ key,
                           const uint64_t* __restrict__ payload, const int32_t* __restrict__ z_start,
                           const int32_t* __restrict__ grp_start, int32_t* __restrict__ MAPZ,
                           int32_t* __restrict__ MAPX, int32_t* __restrict__ MAPY, V* __restrict__ MAPV) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= nnz) return;
    const KeyT k = key[i];
    const uint64_t pl = payload[i];
    const int64_t z = (int64_t)per_z.div(k);
    const int32_t x = (int32_t)((uint64_t)k - (uint64_t)z * per_z.d);
    const int32_t y = (int32_t)(pl >> 32);
    const int32_t first = z_start[z];
    const int32_t rank = (int32_t)(i - first);
    const int32_t occ = z_start[z + 1] - first;
    const int64_t grp = (int64_t)grp_start[z] + rank / g;
    const int32_t slot = rank % g;
    const int64_t dst = grp * g + slot;
    MAPX[dst] = x;
    MAPY[dst] = y;
    MAPV[dst] = (V)pl;
    if (slot == 0) MAPZ[grp] = (int32_t)z;
    if (rank == occ - 1) {  // last entry of its offset: pad the rest of the group
        for (int32_t q = slot + 1; q < g; ++q) {
            MAPX[grp * g + q] = x;
            MAPY[grp * g + q] = y;
            MAPV[grp * g + q] = (V)0;
        }
    }
}

// ---- host helpers ---------------------------------------------------------------------------
insum_status scan_exclusive(void* temp, size_t temp_bytes, const int32_t* in, int32_t* out, int64_t n,
                            hipStream_t s) {
    return exclusive_scan_i32(temp, temp_bytes, in, out, n, s);
}

size_t convert_temp_bytes(int64_t nnz, int64_t longest_scan) {
    return std::max(sort_temp_bytes(nnz), scan_temp_bytes(longest_scan));
}

insum_status read_flags(const Flags* d_flags, Flags* h, hipStream_t s) {
    INSUM_HIP_TRY(hipMemcpyAsync(h, d_flags, sizeof(Flags), hipMemcpyDeviceToHost, s));
    INSUM_HIP_TRY(hipStreamSynchronize(s));
    return INSUM_OK;
}

// ---- typed bodies of the entry points (KeyT = uint32_t when every key fits, else uint64_t) ----
struct Buffers {  // carved from the caller's workspace
    Flags* flags;
    int32_t *cnt, *start, *grp_start;  // per row (block row, offset): counts / first entry / first group
    void* key[2];
    void* val[2];
    int32_t *head, *blk_ord;  // block format only
    void* temp;
    size_t temp_bytes;
};

template <typename KeyT, typename V>
insum_status group_sort_and_bounds(const Buffers& b, int64_t M, int64_t K, int64_t nnz, const int32_t* row,
                                   const int32_t* col, const void* val, int32_t g, hipStream_t s,
                                   const KeyT** sorted_key, const V** sorted_val) {
    KeyT* const keys[2] = {static_cast<KeyT*>(b.key[0]), static_cast<KeyT*>(b.key[1])};
    V* const vals[2] = {static_cast<V*>(b.val[0]), static_cast<V*>(b.val[1])};
    hipLaunchKernelGGL((k_group_keys<KeyT, false>), dim3(blocks_for(nnz)), dim3(kThreads), 0, s, M, K, nnz, row,
                       col, keys[0], b.cnt, b.flags);
    INSUM_HIP_TRY(hipGetLastError());
    const int where = radix_sort_pairs<KeyT, V>(b.temp, b.temp_bytes, keys, static_cast<const V*>(val), vals, nnz,
                                                bits_for((uint64_t)M * (uint64_t)K - 1), s);
    if (where < 0) return (insum_status)(-where);
    *sorted_key = keys[where];
    *sorted_val = vals[where];
    hipLaunchKernelGGL(k_row_bounds<KeyT>, dim3(blocks_for(nnz + 1)), dim3(kThreads), 0, s, nnz, M,
                       Divisor((uint64_t)K), *sorted_key, b.start);
    hipLaunchKernelGGL(k_groups_from_bounds, dim3(blocks_for(M + 1)), dim3(kThreads), 0, s, M, b.start, g, b.cnt);
    INSUM_HIP_TRY(hipGetLastError());
    return INSUM_OK;
}

// Everything of insum_coo_to_groupcoo after argument checking.
template <typename KeyT, typename V>
insum_status group_convert(const Buffers& b, int64_t M, int64_t K, int64_t nnz, const int32_t* row,
                           const int32_t* col, const void* val, int32_t g, bool fill, int64_t* num_groups,
                           int32_t* AM, int32_t* AK, void* AV, int64_t capacity_groups, hipStream_t s) {
    insum_status st;
    const KeyT* skey = nullptr;
    const V* sval = nullptr;
    hipLaunchKernelGGL(k_zero_i32, dim3(1), dim3(kThreads), 0, s, reinterpret_cast<int32_t*>(b.flags),
                       (int64_t)(sizeof(Flags) / 4));
    if (!fill) {  // count mode: atomic histogram of the rows, no sort
        hipLaunchKernelGGL(k_zero_i32, dim3(blocks_for(M + 1)), dim3(kThreads), 0, s, b.cnt, M + 1);
        hipLaunchKernelGGL((k_group_keys<KeyT, true>), dim3(blocks_for(nnz)), dim3(kThreads), 0, s, M, K, nnz, row,
                           col, static_cast<KeyT*>(nullptr), b.cnt, b.flags);
        hipLaunchKernelGGL(k_groups_from_counts, dim3(blocks_for(M + 1)), dim3(kThreads), 0, s, M, b.cnt, g);
    } else {
        st = group_sort_and_bounds<KeyT, V>(b, M, K, nnz, row, col, val, g, s, &skey, &sval);
        if (st != INSUM_OK) return st;
    }
    st = scan_exclusive(b.temp, b.temp_bytes, b.cnt, b.grp_start, M + 1, s);
    if (st != INSUM_OK) return st;
    hipLaunchKernelGGL(k_store_total, dim3(1), dim3(1), 0, s, b.grp_start + M, &b.flags->total_a);
    INSUM_HIP_TRY(hipGetLastError());
    Flags h;
    st = read_flags(b.flags, &h, s);
    if (st != INSUM_OK) return st;
    if (h.out_of_range) return INSUM_ERR_OUT_OF_RANGE;
    const int64_t G = h.total_a;
    *num_groups = G;
    if (!fill) return INSUM_OK;
    if (capacity_groups < G) return INSUM_ERR_CAPACITY;
    hipLaunchKernelGGL((k_group_fill<KeyT, V>), dim3(blocks_for(nnz)), dim3(kThreads), 0, s, Divisor((uint64_t)K),
                       nnz, g, skey, sval, b.start, b.grp_start, AM, AK, static_cast<V*>(AV));
    INSUM_HIP_TRY(hipGetLastError());
    INSUM_HIP_TRY(hipStreamSynchronize(s));
    return INSUM_OK;
}

// What a count call of the block conversion leaves at the front of the workspace, so that a
// fill call with the same arguments can go on from the sorted entries instead of sorting again.
struct BlockState {
    uint64_t magic;
    int64_t M, K, nnz, num_blocks;
    const void *row, *col, *val;
    int32_t bM, bK, dt, which;  // which: buffer pair that holds the sorted entries
};
constexpr uint64_t kBlockStateMagic = 0x31544154534b4c42ull;

__global__ void k_store_block_state(BlockState* dst, BlockState v) { *dst = v; }

template <typename KeyT, typename V>
insum_status block_convert(const Buffers& b, BlockState* d_state, bool resume, int resume_which,
                           int64_t resume_blocks, int64_t M, int64_t K, int64_t nnz, const int32_t* row,
                           const int32_t* col, const void* val, insum_dtype dt, int32_t bM, int32_t bK, int32_t g,
                           bool fill, int32_t* g_used, int64_t* num_groups, int32_t* AM, int32_t* AK, void* AV,
                           int64_t capacity_groups, hipStream_t s) {
    const int64_t nbr = M / bM;
    const Divisor per_block((uint64_t)bM * (uint64_t)bK);
    const Divisor blocks_per_row((uint64_t)(K / bK));
    KeyT* const keys[2] = {static_cast<KeyT*>(b.key[0]), static_cast<KeyT*>(b.key[1])};
    V* const vals[2] = {static_cast<V*>(b.val[0]), static_cast<V*>(b.val[1])};
    insum_status st;
    Flags h;
    int where = resume_which;
    int64_t num_blocks = resume_blocks;
    if (!resume) {
        hipLaunchKernelGGL(k_zero_i32, dim3(blocks_for(nbr + 1)), dim3(kThreads), 0, s, b.cnt, nbr + 1);
        hipLaunchKernelGGL(k_zero_i32, dim3(1), dim3(kThreads), 0, s, reinterpret_cast<int32_t*>(b.flags),
                           (int64_t)(sizeof(Flags) / 4));
        hipLaunchKernelGGL(k_block_keys<KeyT>, dim3(blocks_for(nnz)), dim3(kThreads), 0, s, M, K, nnz, bM, bK, row,
                           col, keys[0], b.flags);
        INSUM_HIP_TRY(hipGetLastError());
        where = radix_sort_pairs<KeyT, V>(b.temp, b.temp_bytes, keys, static_cast<const V*>(val), vals, nnz,
                                          bits_for((uint64_t)M * (uint64_t)K - 1), s);
        if (where < 0) return (insum_status)(-where);
        hipLaunchKernelGGL(k_block_heads<KeyT>, dim3(blocks_for(nnz + 1)), dim3(kThreads), 0, s, nnz, per_block,
                           blocks_per_row, (const KeyT*)keys[where], b.head, b.cnt, b.flags);
        st = scan_exclusive(b.temp, b.temp_bytes, b.head, b.blk_ord, nnz + 1, s);
        if (st != INSUM_OK) return st;
        st = scan_exclusive(b.temp, b.temp_bytes, b.cnt, b.start, nbr + 1, s);
        if (st != INSUM_OK) return st;
        hipLaunchKernelGGL(k_store_total, dim3(1), dim3(1), 0, s, b.start + nbr, &b.flags->total_a);
        INSUM_HIP_TRY(hipGetLastError());
        st = read_flags(b.flags, &h, s);
        if (st != INSUM_OK) return st;
        if (h.out_of_range) return INSUM_ERR_OUT_OF_RANGE;
        if (h.duplicate) return INSUM_ERR_DUPLICATE;
        num_blocks = h.total_a;
    }
    if (g == 0) g = insum_default_group_size(num_blocks, nbr);
    *g_used = g;

    // groups per block row from the block counts (start[] holds their prefix sums)
    hipLaunchKernelGGL(k_groups_from_bounds, dim3(blocks_for(nbr + 1)), dim3(kThreads), 0, s, nbr, b.start, g, b.cnt);
    st = scan_exclusive(b.temp, b.temp_bytes, b.cnt, b.grp_start, nbr + 1, s);
    if (st != INSUM_OK) return st;
    hipLaunchKernelGGL(k_store_total, dim3(1), dim3(1), 0, s, b.grp_start + nbr, &b.flags->total_b);
    if (!fill) {
        BlockState v{};
        v.magic = kBlockStateMagic;
        v.M = M; v.K = K; v.nnz = nnz; v.num_blocks = num_blocks;
        v.row = row; v.col = col; v.val = val;
        v.bM = bM; v.bK = bK; v.dt = (int32_t)dt; v.which = where;
        hipLaunchKernelGGL(k_store_block_state, dim3(1), dim3(1), 0, s, d_state, v);
    }
    INSUM_HIP_TRY(hipGetLastError());
    st = read_flags(b.flags, &h, s);
    if (st != INSUM_OK) return st;
    const int64_t G = h.total_b;
    *num_groups = G;
    if (!fill) return INSUM_OK;
    if (capacity_groups < G) return INSUM_ERR_CAPACITY;

    const int64_t av_elems = G * g * (int64_t)bM * bK;
    hipLaunchKernelGGL(k_fill_zero<V>, dim3(blocks_for(av_elems)), dim3(kThreads), 0, s, static_cast<V*>(AV), av_elems);
    hipLaunchKernelGGL((k_block_fill<KeyT, V>), dim3(blocks_for(nnz)), dim3(kThreads), 0, s, per_block,
                       blocks_per_row, nnz, g, (const KeyT*)keys[where], (const V*)vals[where], b.head, b.blk_ord,
                       b.start, b.grp_start, AM, AK, static_cast<V*>(AV));
    // the entries have been consumed: a later fill call must sort again
    hipLaunchKernelGGL(k_zero_i32, dim3(1), dim3(kThreads), 0, s, reinterpret_cast<int32_t*>(d_state), (int64_t)2);
    INSUM_HIP_TRY(hipGetLastError());
    INSUM_HIP_TRY(hipStreamSynchronize(s));
    return INSUM_OK;
}

template <typename KeyT, typename V>
insum_status map_convert(const Buffers& b, int64_t X, int64_t Y, int64_t Z, int64_t nnz, const int32_t* mx,
                         const int32_t* my, const int32_t* mz, const void* mv, int32_t g, bool fill,
                         int64_t* num_groups, int32_t* MAPZ, int32_t* MAPX, int32_t* MAPY, void* MAPV,
                         int64_t capacity_groups, hipStream_t s) {
    const Divisor per_z((uint64_t)X);
    const dim3 grid_nnz(blocks_for(nnz)), block(kThreads);
    KeyT* const keys[2] = {static_cast<KeyT*>(b.key[0]), static_cast<KeyT*>(b.key[1])};
    uint64_t* const pays[2] = {static_cast<uint64_t*>(b.val[0]), static_cast<uint64_t*>(b.val[1])};
    const KeyT* skey = nullptr;
    const uint64_t* spay = nullptr;
    insum_status st;
    hipLaunchKernelGGL(k_zero_i32, dim3(1), block, 0, s, reinterpret_cast<int32_t*>(b.flags),
                       (int64_t)(sizeof(Flags) / 4));
    if (!fill) {
        hipLaunchKernelGGL(k_zero_i32, dim3(blocks_for(Z + 1)), block, 0, s, b.cnt, Z + 1);
        hipLaunchKernelGGL((k_map_keys<KeyT, V, true>), grid_nnz, block, 0, s, X, Y, Z, nnz, mx, my, mz,
                           static_cast<const V*>(nullptr), static_cast<KeyT*>(nullptr),
                           static_cast<uint64_t*>(nullptr), b.cnt, b.flags);
        hipLaunchKernelGGL(k_groups_from_counts, dim3(blocks_for(Z + 1)), block, 0, s, Z, b.cnt, g);
    } else {
        hipLaunchKernelGGL((k_map_keys<KeyT, V, false>), grid_nnz, block, 0, s, X, Y, Z, nnz, mx, my, mz,
                           static_cast<const V*>(mv), keys[0], pays[0], b.cnt, b.flags);
        INSUM_HIP_TRY(hipGetLastError());
        const int where = radix_sort_pairs<KeyT, uint64_t>(b.temp, b.temp_bytes, keys, (const uint64_t*)pays[0], pays,
                                                           nnz, bits_for((uint64_t)Z * (uint64_t)X - 1), s);
        if (where < 0) return (insum_status)(-where);
        skey = keys[where];
        spay = pays[where];
        hipLaunchKernelGGL(k_row_bounds<KeyT>, dim3(blocks_for(nnz + 1)), block, 0, s, nnz, Z, per_z, skey, b.start);
        hipLaunchKernelGGL(k_groups_from_bounds, dim3(blocks_for(Z + 1)), block, 0, s, Z, b.start, g, b.cnt);
    }
    st = scan_exclusive(b.temp, b.temp_bytes, b.cnt, b.grp_start, Z + 1, s);
    if (st != INSUM_OK) return st;
    hipLaunchKernelGGL(k_store_total, dim3(1), dim3(1), 0, s, b.grp_start + Z, &b.flags->total_a);
    INSUM_HIP_TRY(hipGetLastError());
    Flags h;
    st = read_flags(b.flags, &h, s);
    if (st != INSUM_OK) return st;
    if (h.out_of_range) return INSUM_ERR_OUT_OF_RANGE;
    const int64_t G = h.total_a;
    *num_groups = G;
    if (!fill) return INSUM_OK;
    if (capacity_groups < G) return INSUM_ERR_CAPACITY;
    hipLaunchKernelGGL((k_map_fill<KeyT, V>), grid_nnz, block, 0, s, per_z, nnz, g, skey, spay, b.start, b.grp_start,
                       MAPZ, MAPX, MAPY, static_cast<V*>(MAPV));
    INSUM_HIP_TRY(hipGetLastError());
    INSUM_HIP_TRY(hipStreamSynchronize(s));
    return INSUM_OK;
}

// Workspace layout shared by the three conversions: rows = number of rows / block rows / offsets,
// val_bytes = size of one sorted payload, with_heads = the block format's two extra arrays.
size_t conversion_workspace_bytes(int64_t rows, int64_t nnz, size_t val_bytes, bool with_heads) {
    const size_t n1 = (size_t)std::max<int64_t>(nnz, 1);
    size_t b = 512;
    b += align_up(sizeof(BlockState), 256) + align_up(sizeof(Flags), 256);
    b += 3 * align_up((size_t)(rows + 1) * 4, 256);
    b += 2 * align_up(n1 * 8, 256);          // keys, two buffers
    b += 2 * align_up(n1 * val_bytes, 256);  // payloads, two buffers
    if (with_heads) b += 2 * align_up((size_t)(nnz + 1) * 4, 256);
    b += align_up(convert_temp_bytes(nnz, std::max(rows + 1, with_heads ? nnz + 1 : 0)), 256);
    return b;
}

bool carve(Carver& ws, Buffers& b, BlockState** state, int64_t rows, int64_t nnz, size_t val_bytes,
           bool with_heads) {
    *state = ws.take<BlockState>(1);
    b.flags = ws.take<Flags>(1);
    b.cnt = ws.take<int32_t>(rows + 1);
    b.start = ws.take<int32_t>(rows + 1);
    b.grp_start = ws.take<int32_t>(rows + 1);
    b.key[0] = ws.take<uint64_t>(nnz);
    b.key[1] = ws.take<uint64_t>(nnz);
    b.val[0] = ws.take<char>((size_t)std::max<int64_t>(nnz, 1) * val_bytes);
    b.val[1] = ws.take<char>((size_t)std::max<int64_t>(nnz, 1) * val_bytes);
    b.head = with_heads ? ws.take<int32_t>(nnz + 1) : nullptr;
    b.blk_ord = with_heads ? ws.take<int32_t>(nnz + 1) : nullptr;
    b.temp_bytes = convert_temp_bytes(nnz, std::max(rows + 1, with_heads ? nnz + 1 : 0));
    b.temp = ws.take<char>(b.temp_bytes);
    return ws.ok;
}

}  // namespace
}  // namespace insum

using namespace insum;

// ============================================================================================
extern "C" size_t insum_coo_to_groupcoo_workspace_bytes(int64_t M, int64_t nnz) {
    return conversion_workspace_bytes(std::max<int64_t>(M, 0), std::max<int64_t>(nnz, 0), 4, false);
}

extern "C" insum_status insum_coo_to_groupcoo(int64_t M, int64_t K, int64_t nnz, const int32_t* row,
                                              const int32_t* col, const void* val, insum_dtype dt,
                                              int32_t g, int32_t* g_used, int64_t* num_groups,
                                              int32_t* AM, int32_t* AK, void* AV,
                                              int64_t capacity_groups, void* workspace,
                                              size_t workspace_bytes, void* stream) {
    if (M < 0 || K < 0 || nnz < 0 || g < 0 || !g_used || !num_groups) return INSUM_ERR_INVALID_ARG;
    if (M >= (1LL << 31) || K >= (1LL << 31) || nnz >= (1LL << 31)) return INSUM_ERR_INVALID_ARG;
    if (!dtype_valid(dt)) return INSUM_ERR_INVALID_ARG;
    if (nnz > 0 && (!row || !col || !val)) return INSUM_ERR_INVALID_ARG;
    const bool fill = AM || AK || AV;
    if (fill && (!AM || !AK || !AV || capacity_groups < 0)) return INSUM_ERR_INVALID_ARG;
    if (g == 0) g = insum_default_group_size(nnz, M);
    *g_used = g;
    *num_groups = 0;
    if (nnz == 0) return INSUM_OK;
    if (M == 0 || K == 0) return INSUM_ERR_OUT_OF_RANGE;
    hipStream_t s = static_cast<hipStream_t>(stream);

    Carver ws(workspace, workspace_bytes);
    Buffers b;
    BlockState* unused = nullptr;
    if (!carve(ws, b, &unused, M, nnz, 4, false)) return INSUM_ERR_CAPACITY;
    const bool narrow = bits_for((uint64_t)M * (uint64_t)K - 1) <= 32;
    const bool wide_val = dtype_size(dt) == 4;
#define INSUM_GROUP_CASE(KeyT, V) \
    return group_convert<KeyT, V>(b, M, K, nnz, row, col, val, g, fill, num_groups, AM, AK, AV, capacity_groups, s)
    if (narrow && wide_val) INSUM_GROUP_CASE(uint32_t, uint32_t);
    if (narrow) INSUM_GROUP_CASE(uint32_t, uint16_t);
    if (wide_val) INSUM_GROUP_CASE(uint64_t, uint32_t);
    INSUM_GROUP_CASE(uint64_t, uint16_t);
#undef INSUM_GROUP_CASE
}

// ============================================================================================
namespace {

struct TransposeBuffers {
    int32_t *real, *offs, *row, *col;
    void* val;
    void* scan_temp;
    size_t scan_bytes;
};

size_t transpose_front_bytes(int64_t slots) {   // everything ahead of the conversion's own workspace
    const size_t n1 = (size_t)std::max<int64_t>(slots, 1);
    return 256 + 2 * align_up((n1 + 1) * 4, 256) + 3 * align_up(n1 * 4, 256) +
           align_up(scan_temp_bytes(slots + 1), 256);
}

bool carve_transpose(Carver& ws, TransposeBuffers& t, int64_t slots) {
    t.real = ws.take<int32_t>(slots + 1);
    t.offs = ws.take<int32_t>(slots + 1);
    t.row = ws.take<int32_t>(slots);
    t.col = ws.take<int32_t>(slots);
    t.val = ws.take<int32_t>(slots);   // values are at most 4 bytes wide
    t.scan_bytes = scan_temp_bytes(slots + 1);
    t.scan_temp = ws.take<char>(t.scan_bytes);
    return ws.ok;
}

// the entries of A^T as COO arrays in the workspace; *nnz = their number (synchronises)
template <typename V>
insum_status transposed_entries(const TransposeBuffers& t, int64_t slots, int32_t g, const int32_t* AM,
                                const int32_t* AK, const void* AV, int64_t* nnz, hipStream_t s) {
    const V* av = static_cast<const V*>(AV);
    hipLaunchKernelGGL(k_real_slots<V>, dim3(blocks_for(slots + 1)), dim3(kThreads), 0, s, slots, g, AK, av, t.real);
    INSUM_HIP_TRY(hipGetLastError());
    const insum_status st = scan_exclusive(t.scan_temp, t.scan_bytes, t.real, t.offs, slots + 1, s);
    if (st != INSUM_OK) return st;
    hipLaunchKernelGGL(k_transposed_entries<V>, dim3(blocks_for(slots)), dim3(kThreads), 0, s, slots, g, AM, AK, av,
                       t.offs, t.row, t.col, static_cast<V*>(t.val));
    INSUM_HIP_TRY(hipGetLastError());
    int32_t total = 0;
    INSUM_HIP_TRY(hipMemcpyAsync(&total, t.offs + slots, sizeof(total), hipMemcpyDeviceToHost, s));
    INSUM_HIP_TRY(hipStreamSynchronize(s));
    *nnz = total;
    return INSUM_OK;
}

}  // namespace

extern "C" size_t insum_groupcoo_transpose_workspace_bytes(int64_t M, int64_t K, int64_t G, int32_t g) {
    if (M < 0 || K < 0 || G < 0 || g <= 0 || G >= (1LL << 31) || G * (int64_t)g >= (1LL << 31)) return 0;
    const int64_t slots = G * (int64_t)g;
    return transpose_front_bytes(slots) + insum_coo_to_groupcoo_workspace_bytes(K, slots);
}

extern "C" insum_status insum_groupcoo_transpose(int64_t M, int64_t K, int64_t G, int32_t g, const int32_t* AM,
                                                 const int32_t* AK, const void* AV, insum_dtype dt, int32_t g_t,
                                                 int32_t* g_used, int64_t* num_groups, int64_t* num_entries,
                                                 int32_t* AM_t, int32_t* AK_t, void* AV_t,
                                                 int64_t capacity_groups, void* workspace,
                                                 size_t workspace_bytes, void* stream) {
    if (M < 0 || K < 0 || G < 0 || g <= 0 || g_t < 0 || !g_used || !num_groups) return INSUM_ERR_INVALID_ARG;
    if (M >= (1LL << 31) || K >= (1LL << 31) || G >= (1LL << 31) || G * (int64_t)g >= (1LL << 31))
        return INSUM_ERR_INVALID_ARG;
    if (!dtype_valid(dt)) return INSUM_ERR_INVALID_ARG;
    if (G > 0 && (!AM || !AK || !AV)) return INSUM_ERR_INVALID_ARG;
    const int64_t slots = G * (int64_t)g;
    int64_t nnz = 0;
    Carver ws(workspace, workspace_bytes);
    TransposeBuffers t{};
    if (slots > 0) {
        if (!carve_transpose(ws, t, slots)) return INSUM_ERR_CAPACITY;
        hipStream_t s = static_cast<hipStream_t>(stream);
        const insum_status st = dtype_size(dt) == 4
                                    ? transposed_entries<uint32_t>(t, slots, g, AM, AK, AV, &nnz, s)
                                    : transposed_entries<uint16_t>(t, slots, g, AM, AK, AV, &nnz, s);
        if (st != INSUM_OK) return st;
    }
    if (num_entries) *num_entries = nnz;
    // the rest of the workspace serves the conversion of the exchanged coordinates
    const uintptr_t rest = std::min(ws.cur, ws.end);
    return insum_coo_to_groupcoo(K, M, nnz, t.row, t.col, t.val, dt, g_t, g_used, num_groups, AM_t, AK_t, AV_t,
                                 capacity_groups, reinterpret_cast<void*>(rest), ws.end - rest, stream);
}

// ============================================================================================
extern "C" size_t insum_coo_to_blockgroupcoo_workspace_bytes(int64_t M, int64_t K, int64_t nnz,
                                                             int32_t bM, int32_t bK) {
    (void)K;
    (void)bK;
    M = std::max<int64_t>(M, 0);
    return conversion_workspace_bytes(bM > 0 ? M / bM : M, std::max<int64_t>(nnz, 0), 4, true);
}

extern "C" insum_status insum_coo_to_blockgroupcoo(int64_t M, int64_t K, int64_t nnz,
                                                   const int32_t* row, const int32_t* col,
                                                   const void* val, insum_dtype dt, int32_t bM,
                                                   int32_t bK, int32_t g, int32_t* g_used,
                                                   int64_t* num_groups, int32_t* AM, int32_t* AK,
                                                   void* AV, int64_t capacity_groups,
                                                   void* workspace, size_t workspace_bytes,
                                                   void* stream) {
    if (M < 0 || K < 0 || nnz < 0 || g < 0 || !g_used || !num_groups) return INSUM_ERR_INVALID_ARG;
    if (M >= (1LL << 31) || K >= (1LL << 31) || nnz >= (1LL << 31)) return INSUM_ERR_INVALID_ARG;
    if (!dtype_valid(dt) || bM <= 0 || bK <= 0) return INSUM_ERR_INVALID_ARG;
    if (M % bM || K % bK) return INSUM_ERR_UNSUPPORTED;
    if (nnz > 0 && (!row || !col || !val)) return INSUM_ERR_INVALID_ARG;
    const bool fill = AM || AK || AV;
    if (fill && (!AM || !AK || !AV || capacity_groups < 0)) return INSUM_ERR_INVALID_ARG;
    *g_used = g ? g : 1;
    *num_groups = 0;
    if (nnz == 0) return INSUM_OK;
    if (M == 0 || K == 0) return INSUM_ERR_OUT_OF_RANGE;
    hipStream_t s = static_cast<hipStream_t>(stream);

    Carver ws(workspace, workspace_bytes);
    Buffers b;
    BlockState* d_state = nullptr;
    if (!carve(ws, b, &d_state, M / bM, nnz, 4, true)) return INSUM_ERR_CAPACITY;

    // A fill call right after a count call with the same arguments finds that call's sorted
    // entries, block ordinals and block-row bounds still in the workspace.
    bool resume = false;
    BlockState st{};
    if (fill) {
        INSUM_HIP_TRY(hipMemcpyAsync(&st, d_state, sizeof(st), hipMemcpyDeviceToHost, s));
        INSUM_HIP_TRY(hipStreamSynchronize(s));
        resume = st.magic == kBlockStateMagic && st.M == M && st.K == K && st.nnz == nnz && st.row == row &&
                 st.col == col && st.val == val && st.bM == bM && st.bK == bK && st.dt == (int32_t)dt &&
                 (st.which == 0 || st.which == 1);
    }
    const bool narrow = bits_for((uint64_t)M * (uint64_t)K - 1) <= 32;
    const bool wide_val = dtype_size(dt) == 4;
#define INSUM_BLOCK_CASE(KeyT, V)                                                                              \
    return block_convert<KeyT, V>(b, d_state, resume, st.which, st.num_blocks, M, K, nnz, row, col, val, dt, bM, bK, \
                                  g, fill, g_used, num_groups, AM, AK, AV, capacity_groups, s)
    if (narrow && wide_val) INSUM_BLOCK_CASE(uint32_t, uint32_t);
    if (narrow) INSUM_BLOCK_CASE(uint32_t, uint16_t);
    if (wide_val) INSUM_BLOCK_CASE(uint64_t, uint32_t);
    INSUM_BLOCK_CASE(uint64_t, uint16_t);
#undef INSUM_BLOCK_CASE
}

// ============================================================================================
extern "C" size_t insum_map_to_groupcoo_workspace_bytes(int64_t Z, int64_t nnz) {
    return conversion_workspace_bytes(std::max<int64_t>(Z, 0), std::max<int64_t>(nnz, 0), 8, false);
}

extern "C" insum_status insum_map_to_groupcoo(int64_t X, int64_t Y, int64_t Z, int64_t nnz,
                                              const int32_t* mx, const int32_t* my, const int32_t* mz,
                                              const void* mv, insum_dtype dt, int32_t g, int32_t* g_used,
                                              int64_t* num_groups, int32_t* MAPZ, int32_t* MAPX,
                                              int32_t* MAPY, void* MAPV, int64_t capacity_groups,
                                              void* workspace, size_t workspace_bytes, void* stream) {
    if (X < 0 || Y < 0 || Z < 0 || nnz < 0 || g < 0 || !g_used || !num_groups) return INSUM_ERR_INVALID_ARG;
    if (X >= (1LL << 31) || Y >= (1LL << 31) || Z >= (1LL << 31) || nnz >= (1LL << 31))
        return INSUM_ERR_INVALID_ARG;
    if (!dtype_valid(dt)) return INSUM_ERR_INVALID_ARG;
    if (nnz > 0 && (!mx || !my || !mz || !mv)) return INSUM_ERR_INVALID_ARG;
    const bool fill = MAPZ || MAPX || MAPY || MAPV;
    if (fill && (!MAPZ || !MAPX || !MAPY || !MAPV || capacity_groups < 0)) return INSUM_ERR_INVALID_ARG;
    if (g == 0) g = insum_default_group_size(nnz, Z);
    *g_used = g;
    *num_groups = 0;
    if (nnz == 0) return INSUM_OK;
    if (X == 0 || Y == 0 || Z == 0) return INSUM_ERR_OUT_OF_RANGE;
    hipStream_t s = static_cast<hipStream_t>(stream);

    Carver ws(workspace, workspace_bytes);
    Buffers b;
    BlockState* unused = nullptr;
    if (!carve(ws, b, &unused, Z, nnz, 8, false)) return INSUM_ERR_CAPACITY;
    const bool narrow = bits_for((uint64_t)Z * (uint64_t)X - 1) <= 32;
    const bool wide_val = dtype_size(dt) == 4;
#define INSUM_MAP_CASE(KeyT, V)                                                                             \
    return map_convert<KeyT, V>(b, X, Y, Z, nnz, mx, my, mz, mv, g, fill, num_groups, MAPZ, MAPX, MAPY, MAPV, \
                                capacity_groups, s)
    if (narrow && wide_val) INSUM_MAP_CASE(uint32_t, uint32_t);
    if (narrow) INSUM_MAP_CASE(uint32_t, uint16_t);
    if (wide_val) INSUM_MAP_CASE(uint64_t, uint32_t);
    INSUM_MAP_CASE(uint64_t, uint16_t);
#undef INSUM_MAP_CASE
}
