// COO -> GroupCOO and COO -> BlockGroupCOO on the device (paper: Section 4.1).
//
// The paper fixes the result (fixed-length groups along rows / block rows, the row stored
// once per group, padding inside a row's last group) but not an algorithm.  Here:
//   1. one pass validates coordinates, counts entries per row and forms a 64-bit sort key
//      (GroupCOO: row*K + col; blocks: ((block row, block col), position inside block));
//   2. a stable radix sort of (key, input position) gives the canonical order
//      (row, col, input position);
//   3. prefix sums of ceil(occ/g) give each row's first group; G goes back to the host;
//   4. one pass scatters every sorted entry to group = first_group[row] + rank/g,
//      slot = rank % g, and the last entry of a row also writes that group's padding.
// Values are moved as raw bits; there is no floating-point arithmetic, so the output is a
// pure function of the input.
//
// The device-wide sort and prefix sums are rocPRIM's (library primitives); everything
// specific to the formats is in the kernels of this file.
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_scan.hpp>

#include <algorithm>

#include "common.h"

namespace insum {
namespace {

constexpr int kThreads = 256;

inline unsigned blocks_for(int64_t n) { return (unsigned)std::max<int64_t>(1, ceil_div(n, kThreads)); }

int bits_for(uint64_t max_value) {  // number of low bits that can be set in [0, max_value]
    int b = 0;
    while (b < 64 && (max_value >> b) != 0) ++b;
    return std::max(b, 1);
}

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

size_t sort_temp_bytes(int64_t nnz) {
    size_t bytes = 0;
    uint64_t* k = nullptr;
    uint32_t* v = nullptr;
    (void)rocprim::radix_sort_pairs(nullptr, bytes, k, k, v, v, (size_t)std::max<int64_t>(nnz, 1), 0, 64);
    return bytes;
}

size_t scan_temp_bytes(int64_t n) {
    size_t bytes = 0;
    int32_t* x = nullptr;
    (void)rocprim::exclusive_scan(nullptr, bytes, x, x, 0, (size_t)std::max<int64_t>(n, 1),
                                  rocprim::plus<int32_t>());
    return bytes;
}

struct Flags {  // device-side status words, copied to the host with the counts
    int32_t out_of_range;
    int32_t duplicate;
    int32_t total_a;  // GroupCOO: G.  Blocks: number of nonzero blocks
    int32_t total_b;  // Blocks: G
};

// ---- kernels: GroupCOO ---------------------------------------------------------------------
__global__ void k_zero_i32(int32_t* p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) p[i] = 0;
}

__global__ void k_group_keys(int64_t M, int64_t K, int64_t nnz, const int32_t* __restrict__ row,
                             const int32_t* __restrict__ col, uint64_t* __restrict__ key,
                             uint32_t* __restrict__ pos, int32_t* __restrict__ occ, Flags* flags) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= nnz) return;
    const int32_t r = row[i], c = col[i];
    if (r < 0 || r >= M || c < 0 || c >= K) {
        flags->out_of_range = 1;
        key[i] = 0;
        pos[i] = (uint32_t)i;
        return;
    }
    key[i] = (uint64_t)r * (uint64_t)K + (uint64_t)c;
    pos[i] = (uint32_t)i;
    atomicAdd(&occ[r], 1);
}

// gpr[i] = ceil(occ[i] / g) for i < n, gpr[n] = 0 (so that an exclusive scan over n+1
// elements ends with the total)
__global__ void k_groups_per_row(int64_t n, const int32_t* occ, int32_t g, int32_t* gpr) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i > n) return;
    gpr[i] = i < n ? (occ[i] + g - 1) / g : 0;
}

template <typename V>
__global__ void k_group_fill(int64_t K, int64_t nnz, int32_t g, const uint64_t* __restrict__ key,
                             const uint32_t* __restrict__ pos, const V* __restrict__ val,
                             const int32_t* __restrict__ row_start,
                             const int32_t* __restrict__ grp_start, int32_t* __restrict__ AM,
                             int32_t* __restrict__ AK, V* __restrict__ AV) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= nnz) return;
    const uint64_t k = key[i];
    const int64_t r = (int64_t)(k / (uint64_t)K);
    const int32_t c = (int32_t)(k - (uint64_t)r * (uint64_t)K);
    const int32_t rank = (int32_t)(i - row_start[r]);
    const int32_t occ = row_start[r + 1] - row_start[r];
    const int64_t grp = (int64_t)grp_start[r] + rank / g;
    const int32_t slot = rank % g;
    const int64_t dst = grp * g + slot;
    AK[dst] = c;
    AV[dst] = val[pos[i]];
    if (slot == 0) AM[grp] = (int32_t)r;
    if (rank == occ - 1) {  // last entry of its row: pad the rest of the group
        for (int32_t q = slot + 1; q < g; ++q) {
            AK[grp * g + q] = c;
            AV[grp * g + q] = (V)0;
        }
    }
}

// ---- kernels: BlockGroupCOO ----------------------------------------------------------------
__global__ void k_block_keys(int64_t M, int64_t K, int64_t nnz, int32_t bM, int32_t bK,
                             const int32_t* __restrict__ row, const int32_t* __restrict__ col,
                             uint64_t* __restrict__ key, uint32_t* __restrict__ pos, Flags* flags) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= nnz) return;
    const int32_t r = row[i], c = col[i];
    pos[i] = (uint32_t)i;
    if (r < 0 || r >= M || c < 0 || c >= K) {
        flags->out_of_range = 1;
        key[i] = 0;
        return;
    }
    const uint64_t nbc = (uint64_t)(K / bK);
    const uint64_t blk = (uint64_t)(r / bM) * nbc + (uint64_t)(c / bK);
    key[i] = (blk * (uint64_t)bM + (uint64_t)(r % bM)) * (uint64_t)bK + (uint64_t)(c % bK);
}

// On sorted keys: head[i] = 1 when entry i is the first of its block; counts blocks per
// block row; equal neighbouring keys are duplicate coordinates.  head has nnz+1 entries
// (the last is 0) so its exclusive scan ends with the number of blocks.
__global__ void k_block_heads(int64_t nnz, int64_t K, int32_t bM, int32_t bK,
                              const uint64_t* __restrict__ key, int32_t* __restrict__ head,
                              int32_t* __restrict__ occ, Flags* flags) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i > nnz) return;
    if (i == nnz) {
        head[i] = 0;
        return;
    }
    const uint64_t per_block = (uint64_t)bM * (uint64_t)bK;
    const uint64_t blk = key[i] / per_block;
    int32_t h = 1;
    if (i > 0) {
        const uint64_t prev = key[i - 1];
        if (prev == key[i]) flags->duplicate = 1;
        h = (prev / per_block) != blk;
    }
    head[i] = h;
    if (h) atomicAdd(&occ[blk / (uint64_t)(K / bK)], 1);
}

template <typename V>
__global__ void k_fill_zero(V* p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) p[i] = (V)0;
}

template <typename V>
__global__ void k_block_fill(int64_t K, int64_t nnz, int32_t bM, int32_t bK, int32_t g,
                             const uint64_t* __restrict__ key, const uint32_t* __restrict__ pos,
                             const V* __restrict__ val, const int32_t* __restrict__ head,
                             const int32_t* __restrict__ blk_ord,
                             const int32_t* __restrict__ brow_start,
                             const int32_t* __restrict__ grp_start, int32_t* __restrict__ AM,
                             int32_t* __restrict__ AK, V* __restrict__ AV) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= nnz) return;
    const uint64_t per_block = (uint64_t)bM * (uint64_t)bK;
    const uint64_t nbc = (uint64_t)(K / bK);
    const uint64_t k = key[i];
    const uint64_t blk = k / per_block;
    const uint64_t inside = k - blk * per_block;  // bm * bK + bk
    const int64_t br = (int64_t)(blk / nbc);
    const int32_t bc = (int32_t)(blk - (uint64_t)br * nbc);
    // blk_ord is the exclusive scan of head: for a head entry it is the block's ordinal,
    // for the other entries of the block it is ordinal + 1.
    const int32_t ord = blk_ord[i] - (head[i] ? 0 : 1);
    const int32_t rank = ord - brow_start[br];
    const int32_t occ = brow_start[br + 1] - brow_start[br];
    const int64_t grp = (int64_t)grp_start[br] + rank / g;
    const int32_t slot = rank % g;
    AV[((grp * g + slot) * (int64_t)per_block) + (int64_t)inside] = val[pos[i]];
    if (head[i]) {
        AK[grp * g + slot] = bc;
        if (slot == 0) AM[grp] = (int32_t)br;
        if (rank == occ - 1)
            for (int32_t q = slot + 1; q < g; ++q) AK[grp * g + q] = bc;
    }
}

template <typename T>
insum_status scan_exclusive(void* temp, size_t temp_bytes, const T* in, T* out, int64_t n,
                            hipStream_t s) {
    INSUM_HIP_TRY(rocprim::exclusive_scan(temp, temp_bytes, in, out, (T)0, (size_t)n,
                                          rocprim::plus<T>(), s));
    return INSUM_OK;
}

insum_status read_flags(const Flags* d_flags, Flags* h, hipStream_t s) {
    INSUM_HIP_TRY(hipMemcpyAsync(h, d_flags, sizeof(Flags), hipMemcpyDeviceToHost, s));
    INSUM_HIP_TRY(hipStreamSynchronize(s));
    return INSUM_OK;
}

__global__ void k_store_total(const int32_t* src, int32_t* dst) { *dst = *src; }

}  // namespace
}  // namespace insum

using namespace insum;

// ============================================================================================
extern "C" size_t insum_coo_to_groupcoo_workspace_bytes(int64_t M, int64_t nnz) {
    M = std::max<int64_t>(M, 0);
    nnz = std::max<int64_t>(nnz, 0);
    size_t b = 512;
    b += align_up(sizeof(Flags), 256);
    b += 3 * align_up((size_t)(M + 1) * 4, 256);            // occ / groups-per-row, row_start, grp_start
    b += 2 * align_up((size_t)std::max<int64_t>(nnz, 1) * 8, 256);  // keys in/out
    b += 2 * align_up((size_t)std::max<int64_t>(nnz, 1) * 4, 256);  // positions in/out
    b += align_up(std::max(sort_temp_bytes(nnz), scan_temp_bytes(M + 1)), 256);
    return b;
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
    Flags* d_flags = ws.take<Flags>(1);
    int32_t* occ = ws.take<int32_t>(M + 1);  // later reused for groups per row
    int32_t* row_start = ws.take<int32_t>(M + 1);
    int32_t* grp_start = ws.take<int32_t>(M + 1);
    uint64_t* key_a = ws.take<uint64_t>(nnz);
    uint64_t* key_b = ws.take<uint64_t>(nnz);
    uint32_t* pos_a = ws.take<uint32_t>(nnz);
    uint32_t* pos_b = ws.take<uint32_t>(nnz);
    const size_t temp_bytes = std::max(sort_temp_bytes(nnz), scan_temp_bytes(M + 1));
    void* temp = ws.take<char>(temp_bytes);
    if (!ws.ok) return INSUM_ERR_CAPACITY;

    hipLaunchKernelGGL(k_zero_i32, dim3(blocks_for(M + 1)), dim3(kThreads), 0, s, occ, M + 1);
    hipLaunchKernelGGL(k_zero_i32, dim3(1), dim3(kThreads), 0, s, reinterpret_cast<int32_t*>(d_flags),
                       (int64_t)(sizeof(Flags) / 4));
    hipLaunchKernelGGL(k_group_keys, dim3(blocks_for(nnz)), dim3(kThreads), 0, s, M, K, nnz, row, col,
                       key_a, pos_a, occ, d_flags);
    insum_status st = scan_exclusive(temp, temp_bytes, occ, row_start, M + 1, s);
    if (st != INSUM_OK) return st;
    hipLaunchKernelGGL(k_groups_per_row, dim3(blocks_for(M + 1)), dim3(kThreads), 0, s, M, occ, g, occ);
    st = scan_exclusive(temp, temp_bytes, occ, grp_start, M + 1, s);
    if (st != INSUM_OK) return st;
    hipLaunchKernelGGL(k_store_total, dim3(1), dim3(1), 0, s, grp_start + M, &d_flags->total_a);
    INSUM_HIP_TRY(hipGetLastError());
    Flags h;
    st = read_flags(d_flags, &h, s);
    if (st != INSUM_OK) return st;
    if (h.out_of_range) return INSUM_ERR_OUT_OF_RANGE;
    const int64_t G = h.total_a;
    *num_groups = G;
    if (!fill) return INSUM_OK;
    if (capacity_groups < G) return INSUM_ERR_CAPACITY;

    const int key_bits = bits_for((uint64_t)M * (uint64_t)K - 1);
    size_t tb = 0;
    INSUM_HIP_TRY(rocprim::radix_sort_pairs(nullptr, tb, key_a, key_b, pos_a, pos_b, (size_t)nnz, 0,
                                            key_bits, s));
    if (tb > temp_bytes) return INSUM_ERR_CAPACITY;
    INSUM_HIP_TRY(rocprim::radix_sort_pairs(temp, tb, key_a, key_b, pos_a, pos_b, (size_t)nnz, 0,
                                            key_bits, s));
    if (dtype_size(dt) == 4)
        hipLaunchKernelGGL(k_group_fill<uint32_t>, dim3(blocks_for(nnz)), dim3(kThreads), 0, s, K, nnz, g,
                           key_b, pos_b, static_cast<const uint32_t*>(val), row_start, grp_start, AM, AK,
                           static_cast<uint32_t*>(AV));
    else
        hipLaunchKernelGGL(k_group_fill<uint16_t>, dim3(blocks_for(nnz)), dim3(kThreads), 0, s, K, nnz, g,
                           key_b, pos_b, static_cast<const uint16_t*>(val), row_start, grp_start, AM, AK,
                           static_cast<uint16_t*>(AV));
    INSUM_HIP_TRY(hipGetLastError());
    INSUM_HIP_TRY(hipStreamSynchronize(s));
    return INSUM_OK;
}

// ============================================================================================
extern "C" size_t insum_coo_to_blockgroupcoo_workspace_bytes(int64_t M, int64_t K, int64_t nnz,
                                                             int32_t bM, int32_t bK) {
    (void)K;
    (void)bK;
    M = std::max<int64_t>(M, 0);
    nnz = std::max<int64_t>(nnz, 0);
    const int64_t nbr = bM > 0 ? M / bM : M;
    size_t b = 512;
    b += align_up(sizeof(Flags), 256);
    b += 3 * align_up((size_t)(nbr + 1) * 4, 256);           // occ, brow_start, grp_start
    b += 2 * align_up((size_t)std::max<int64_t>(nnz, 1) * 8, 256);   // keys in/out
    b += 2 * align_up((size_t)std::max<int64_t>(nnz, 1) * 4, 256);   // positions in/out
    b += 2 * align_up((size_t)(nnz + 1) * 4, 256);           // head flags, block ordinals
    b += align_up(std::max({sort_temp_bytes(nnz), scan_temp_bytes(nnz + 1), scan_temp_bytes(nbr + 1)}), 256);
    return b;
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
    const int64_t nbr = M / bM;
    *g_used = g ? g : 1;
    *num_groups = 0;
    if (nnz == 0) return INSUM_OK;
    if (M == 0 || K == 0) return INSUM_ERR_OUT_OF_RANGE;
    hipStream_t s = static_cast<hipStream_t>(stream);

    Carver ws(workspace, workspace_bytes);
    Flags* d_flags = ws.take<Flags>(1);
    int32_t* occ = ws.take<int32_t>(nbr + 1);
    int32_t* brow_start = ws.take<int32_t>(nbr + 1);
    int32_t* grp_start = ws.take<int32_t>(nbr + 1);
    uint64_t* key_a = ws.take<uint64_t>(nnz);
    uint64_t* key_b = ws.take<uint64_t>(nnz);
    uint32_t* pos_a = ws.take<uint32_t>(nnz);
    uint32_t* pos_b = ws.take<uint32_t>(nnz);
    int32_t* head = ws.take<int32_t>(nnz + 1);
    int32_t* blk_ord = ws.take<int32_t>(nnz + 1);
    const size_t temp_bytes =
        std::max({sort_temp_bytes(nnz), scan_temp_bytes(nnz + 1), scan_temp_bytes(nbr + 1)});
    void* temp = ws.take<char>(temp_bytes);
    if (!ws.ok) return INSUM_ERR_CAPACITY;

    hipLaunchKernelGGL(k_zero_i32, dim3(blocks_for(nbr + 1)), dim3(kThreads), 0, s, occ, nbr + 1);
    hipLaunchKernelGGL(k_zero_i32, dim3(1), dim3(kThreads), 0, s, reinterpret_cast<int32_t*>(d_flags),
                       (int64_t)(sizeof(Flags) / 4));
    hipLaunchKernelGGL(k_block_keys, dim3(blocks_for(nnz)), dim3(kThreads), 0, s, M, K, nnz, bM, bK, row,
                       col, key_a, pos_a, d_flags);
    INSUM_HIP_TRY(hipGetLastError());
    const int key_bits = bits_for((uint64_t)M * (uint64_t)K - 1);
    size_t tb = 0;
    INSUM_HIP_TRY(rocprim::radix_sort_pairs(nullptr, tb, key_a, key_b, pos_a, pos_b, (size_t)nnz, 0,
                                            key_bits, s));
    if (tb > temp_bytes) return INSUM_ERR_CAPACITY;
    INSUM_HIP_TRY(rocprim::radix_sort_pairs(temp, tb, key_a, key_b, pos_a, pos_b, (size_t)nnz, 0,
                                            key_bits, s));
    hipLaunchKernelGGL(k_block_heads, dim3(blocks_for(nnz + 1)), dim3(kThreads), 0, s, nnz, K, bM, bK,
                       key_b, head, occ, d_flags);
    insum_status st = scan_exclusive(temp, temp_bytes, head, blk_ord, nnz + 1, s);
    if (st != INSUM_OK) return st;
    st = scan_exclusive(temp, temp_bytes, occ, brow_start, nbr + 1, s);
    if (st != INSUM_OK) return st;
    hipLaunchKernelGGL(k_store_total, dim3(1), dim3(1), 0, s, brow_start + nbr, &d_flags->total_a);
    INSUM_HIP_TRY(hipGetLastError());
    Flags h;
    st = read_flags(d_flags, &h, s);
    if (st != INSUM_OK) return st;
    if (h.out_of_range) return INSUM_ERR_OUT_OF_RANGE;
    if (h.duplicate) return INSUM_ERR_DUPLICATE;
    const int64_t num_blocks = h.total_a;
    if (g == 0) g = insum_default_group_size(num_blocks, nbr);
    *g_used = g;

    hipLaunchKernelGGL(k_groups_per_row, dim3(blocks_for(nbr + 1)), dim3(kThreads), 0, s, nbr, occ, g, occ);
    st = scan_exclusive(temp, temp_bytes, occ, grp_start, nbr + 1, s);
    if (st != INSUM_OK) return st;
    hipLaunchKernelGGL(k_store_total, dim3(1), dim3(1), 0, s, grp_start + nbr, &d_flags->total_b);
    INSUM_HIP_TRY(hipGetLastError());
    st = read_flags(d_flags, &h, s);
    if (st != INSUM_OK) return st;
    const int64_t G = h.total_b;
    *num_groups = G;
    if (!fill) return INSUM_OK;
    if (capacity_groups < G) return INSUM_ERR_CAPACITY;

    const int64_t av_elems = G * g * (int64_t)bM * bK;
    if (dtype_size(dt) == 4) {
        hipLaunchKernelGGL(k_fill_zero<uint32_t>, dim3(blocks_for(av_elems)), dim3(kThreads), 0, s,
                           static_cast<uint32_t*>(AV), av_elems);
        hipLaunchKernelGGL(k_block_fill<uint32_t>, dim3(blocks_for(nnz)), dim3(kThreads), 0, s, K, nnz, bM,
                           bK, g, key_b, pos_b, static_cast<const uint32_t*>(val), head, blk_ord, brow_start,
                           grp_start, AM, AK, static_cast<uint32_t*>(AV));
    } else {
        hipLaunchKernelGGL(k_fill_zero<uint16_t>, dim3(blocks_for(av_elems)), dim3(kThreads), 0, s,
                           static_cast<uint16_t*>(AV), av_elems);
        hipLaunchKernelGGL(k_block_fill<uint16_t>, dim3(blocks_for(nnz)), dim3(kThreads), 0, s, K, nnz, bM,
                           bK, g, key_b, pos_b, static_cast<const uint16_t*>(val), head, blk_ord, brow_start,
                           grp_start, AM, AK, static_cast<uint16_t*>(AV));
    }
    INSUM_HIP_TRY(hipGetLastError());
    INSUM_HIP_TRY(hipStreamSynchronize(s));
    return INSUM_OK;
}
