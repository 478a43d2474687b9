// Device-wide primitives of the format conversions, written for 64-lane wavefronts:
//   * exclusive prefix sums of int32 arrays (reduce / scan of the block sums / scan with carry-in,
//     recursive in the number of blocks);
//   * a stable least-significant-digit radix sort of (key, value) pairs, 8 bits per pass:
//     per-tile digit counts -> prefix sums over (digit, tile) -> stable scatter.  Only as many
//     passes run as the largest possible key has digits.
// The conversions need the canonical order (row, column, input position) of Section 4.1's
// formats bit for bit: equal keys must keep their input order, which is what "stable" buys.
// Everything is enqueued on the caller's stream; nothing here synchronises or allocates.
#pragma once

#include <algorithm>

#include "common.h"

namespace insum {

constexpr int kScanThreads = 256;
constexpr int kScanItems = 16;
constexpr int kScanTile = kScanThreads * kScanItems;  // elements per workgroup

typedef int32_t i32x4 __attribute__((ext_vector_type(4)));

// Exclusive prefix sum of one value per thread over a workgroup of kScanThreads threads;
// *total receives the sum of all values.  `wave_sums` is LDS, one int per wavefront.
__device__ inline int32_t block_exclusive_scan(int32_t v, int32_t* wave_sums, int32_t* total) {
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    int32_t incl = v;
#pragma unroll
    for (int d = 1; d < 64; d *= 2) {
        const int32_t up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    __syncthreads();  // wave_sums may still be in use by an earlier call
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    int32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / 64; ++w) {
        const int32_t s = wave_sums[w];
        if (w < wave) before += s;
        all += s;
    }
    *total = all;
    return before + incl - v;
}

// Thread t of a workgroup owns elements [t*kScanItems, (t+1)*kScanItems) of the tile.
__device__ inline void load_tile(const int32_t* __restrict__ in, int64_t base, int64_t n, int32_t (&x)[kScanItems]) {
    const int64_t first = base + (int64_t)threadIdx.x * kScanItems;
    if (first + kScanItems <= n && (reinterpret_cast<uintptr_t>(in + first) % 16) == 0) {
#pragma unroll
        for (int i = 0; i < kScanItems; i += 4) {
            const i32x4 v = *reinterpret_cast<const i32x4*>(in + first + i);
            x[i] = v.x; x[i + 1] = v.y; x[i + 2] = v.z; x[i + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < kScanItems; ++i) x[i] = first + i < n ? in[first + i] : 0;
    }
}

__global__ __launch_bounds__(kScanThreads) void k_scan_reduce(const int32_t* __restrict__ in, int64_t n,
                                                               int32_t* __restrict__ block_sums) {
    __shared__ int32_t wave_sums[kScanThreads / 64];
    int32_t x[kScanItems];
    load_tile(in, (int64_t)blockIdx.x * kScanTile, n, x);
    int32_t sum = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) sum += x[i];
    int32_t total;
    (void)block_exclusive_scan(sum, wave_sums, &total);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

// out[i] = carry[block] + sum of in[tile start .. i); carry == nullptr: a single tile.  in == out is allowed.
__global__ __launch_bounds__(kScanThreads) void k_scan_tile(const int32_t* in, int32_t* out, int64_t n,
                                                             const int32_t* __restrict__ carry) {
    __shared__ int32_t wave_sums[kScanThreads / 64];
    int32_t x[kScanItems];
    const int64_t base = (int64_t)blockIdx.x * kScanTile;
    load_tile(in, base, n, x);
    int32_t sum = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) sum += x[i];
    int32_t total;
    int32_t run = block_exclusive_scan(sum, wave_sums, &total) + (carry ? carry[blockIdx.x] : 0);
    const int64_t first = base + (int64_t)threadIdx.x * kScanItems;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        if (first + i < n) out[first + i] = run;
        run += x[i];
    }
}

inline int64_t scan_blocks(int64_t n) { return std::max<int64_t>(1, ceil_div(n, kScanTile)); }

// Scratch for the sums of the blocks of every level of the recursion.
inline size_t scan_temp_bytes(int64_t n) {
    size_t bytes = 0;
    for (int64_t m = scan_blocks(n); m > 1; m = scan_blocks(m)) bytes += align_up((size_t)m * sizeof(int32_t), 256);
    return bytes + 256;
}

inline insum_status exclusive_scan_i32(void* temp, size_t temp_bytes, const int32_t* in, int32_t* out,
                                       int64_t n, hipStream_t s) {
    if (n <= 0) return INSUM_OK;
    const int64_t nb = scan_blocks(n);
    if (nb == 1) {
        hipLaunchKernelGGL(k_scan_tile, dim3(1), dim3(kScanThreads), 0, s, in, out, n, (const int32_t*)nullptr);
        INSUM_HIP_TRY(hipGetLastError());
        return INSUM_OK;
    }
    const size_t mine = align_up((size_t)nb * sizeof(int32_t), 256);
    if (!temp || temp_bytes < mine) return INSUM_ERR_CAPACITY;
    int32_t* sums = static_cast<int32_t*>(temp);
    hipLaunchKernelGGL(k_scan_reduce, dim3((unsigned)nb), dim3(kScanThreads), 0, s, in, n, sums);
    const insum_status st = exclusive_scan_i32(static_cast<char*>(temp) + mine, temp_bytes - mine, sums, sums, nb, s);
    if (st != INSUM_OK) return st;
    hipLaunchKernelGGL(k_scan_tile, dim3((unsigned)nb), dim3(kScanThreads), 0, s, in, out, n, (const int32_t*)sums);
    INSUM_HIP_TRY(hipGetLastError());
    return INSUM_OK;
}

// ---- radix sort ------------------------------------------------------------------------------
constexpr int kRadixBits = 8;
constexpr int kRadix = 1 << kRadixBits;
constexpr int kSortThreads = 256;  // four wavefronts; wavefront w owns a contiguous quarter of the tile
static_assert(kSortThreads == kRadix && kScanThreads == kSortThreads, "one thread per digit in the tile kernels");

template <int ITEMS>
struct SortTile {
    static constexpr int kTile = kSortThreads * ITEMS;
    static constexpr int kPerWave = 64 * ITEMS;
};

// table[d * ntiles + t] = number of keys of tile t whose digit is d
template <typename KeyT, int ITEMS>
__global__ __launch_bounds__(kSortThreads) void k_radix_count(const KeyT* __restrict__ keys, int64_t n, int shift,
                                                               int32_t* __restrict__ table, int64_t ntiles) {
    __shared__ int32_t bins[kRadix];
    bins[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * SortTile<ITEMS>::kTile;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int64_t idx = base + (int64_t)i * kSortThreads + threadIdx.x;
        if (idx < n) atomicAdd(&bins[(int)((keys[idx] >> shift) & (kRadix - 1))], 1);
    }
    __syncthreads();
    table[(int64_t)threadIdx.x * ntiles + blockIdx.x] = bins[threadIdx.x];
}

// `table` now holds the exclusive prefix sums of the counts in (digit, tile) order: the first
// output position of the tile's keys with that digit.  The tile is split stably: wavefront w
// walks its quarter of the tile 64 keys at a time; lanes with equal digits find each other with
// eight ballots, so a key's rank among the equal digits of its wavefront is a population count
// plus a running per-wavefront counter; the quarters are then chained in order.  The pairs are
// first placed in LDS in sorted order and written out from there, so that neighbouring lanes
// write neighbouring addresses.
template <typename KeyT, typename ValT, int ITEMS>
__global__ __launch_bounds__(kSortThreads) void k_radix_scatter(const KeyT* __restrict__ keys_in,
                                                                 const ValT* __restrict__ vals_in,
                                                                 KeyT* __restrict__ keys_out,
                                                                 ValT* __restrict__ vals_out, int64_t n, int shift,
                                                                 const int32_t* __restrict__ table, int64_t ntiles) {
    constexpr int TILE = SortTile<ITEMS>::kTile, PER_WAVE = SortTile<ITEMS>::kPerWave, WAVES = kSortThreads / 64;
    __shared__ int32_t count[WAVES][kRadix];  // per wavefront: running count, then offset inside the tile
    __shared__ int32_t delta[kRadix];         // output position minus position in the sorted tile
    __shared__ int32_t wave_sums[WAVES];
    __shared__ KeyT skey[TILE];
    __shared__ ValT sval[TILE];
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    const int64_t base = (int64_t)blockIdx.x * TILE;
    const int tile_n = (int)(n - base < TILE ? n - base : TILE);
#pragma unroll
    for (int w = 0; w < WAVES; ++w) count[w][threadIdx.x] = 0;
    __syncthreads();

    KeyT key[ITEMS];
    ValT val[ITEMS];
    int32_t rank[ITEMS];  // among the keys of this wavefront with the same digit
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int local = wave * PER_WAVE + i * 64 + lane;
        const bool valid = local < tile_n;
        key[i] = valid ? keys_in[base + local] : (KeyT)0;
        val[i] = valid ? vals_in[base + local] : (ValT)0;
    }
    const uint64_t lanes_below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const bool valid = wave * PER_WAVE + i * 64 + lane < tile_n;
        const int d = (int)((key[i] >> shift) & (kRadix - 1));
        uint64_t same = __ballot(valid);
#pragma unroll
        for (int b = 0; b < kRadixBits; ++b) {
            const bool bit = (d >> b) & 1;
            const uint64_t set = __ballot(bit);
            same &= bit ? set : ~set;
        }
        int32_t before = 0;
        // `same`: the valid lanes whose digit equals mine (for a lane past the end of the tile:
        // those with digit 0 - its rank is never used).  The lowest of them advances the counter.
        const int leader = same ? __builtin_ctzll(same) : 0;
        if (valid && lane == leader) {
            before = count[wave][d];
            count[wave][d] = before + __popcll(same);
        }
        before = __shfl(before, leader, 64);
        rank[i] = before + __popcll(same & lanes_below);
    }
    __syncthreads();

    // Thread d: chain the wavefronts' counts of digit d, then place the digits one after the other.
    {
        const int d = threadIdx.x;
        int32_t run = 0;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            const int32_t c = count[w][d];
            count[w][d] = run;
            run += c;
        }
        int32_t total;
        const int32_t start = block_exclusive_scan(run, wave_sums, &total);
#pragma unroll
        for (int w = 0; w < WAVES; ++w) count[w][d] += start;
        delta[d] = table[(int64_t)d * ntiles + blockIdx.x] - start;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        if (wave * PER_WAVE + i * 64 + lane < tile_n) {
            const int d = (int)((key[i] >> shift) & (kRadix - 1));
            const int pos = count[wave][d] + rank[i];
            skey[pos] = key[i];
            sval[pos] = val[i];
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int j = i * kSortThreads + threadIdx.x;
        if (j < tile_n) {
            const KeyT k = skey[j];
            const int64_t dst = (int64_t)delta[(int)((k >> shift) & (kRadix - 1))] + j;
            keys_out[dst] = k;
            vals_out[dst] = sval[j];
        }
    }
}

template <typename KeyT, typename ValT>
struct SortItems {  // keys per thread: 48 KB of staging for 12-byte pairs, 32 KB for 16-byte pairs
    static constexpr int value = sizeof(KeyT) + sizeof(ValT) > 12 ? 8 : 16;
};

template <typename KeyT, typename ValT>
inline int64_t sort_tiles(int64_t n) {
    return std::max<int64_t>(1, ceil_div(n, SortTile<SortItems<KeyT, ValT>::value>::kTile));
}

// Scratch of the sort: the (digit, tile) table and the scan's own scratch.  Sized for the
// smallest tile any instantiation uses.
inline size_t sort_temp_bytes(int64_t n) {
    const int64_t tiles = std::max<int64_t>(1, ceil_div(n, SortTile<8>::kTile));
    return align_up((size_t)tiles * kRadix * sizeof(int32_t), 256) + scan_temp_bytes(tiles * kRadix) + 256;
}

// Sorts n pairs by the low `key_bits` bits of the key, stably.  The pairs start in
// (keys[0], vals_first) and bounce between the two buffer pairs; the return value (0 or 1, or
// a negative status) says which of (keys[i], vals[i]) holds the result.  vals_first is only
// read (by the first pass, which writes vals[1]): it may be a caller-owned read-only array, or
// vals[0] itself; with zero passes the values are copied into vals[0].
template <typename KeyT, typename ValT>
inline int radix_sort_pairs(void* temp, size_t temp_bytes, KeyT* const (&keys)[2], const ValT* vals_first,
                            ValT* const (&vals)[2], int64_t n, int key_bits, hipStream_t s) {
    constexpr int ITEMS = SortItems<KeyT, ValT>::value;
    const int64_t tiles = sort_tiles<KeyT, ValT>(n);
    const size_t table_bytes = align_up((size_t)tiles * kRadix * sizeof(int32_t), 256);
    if (!temp || temp_bytes < table_bytes) return -(int)INSUM_ERR_CAPACITY;
    int32_t* table = static_cast<int32_t*>(temp);
    void* scan_temp = static_cast<char*>(temp) + table_bytes;
    const size_t scan_bytes = temp_bytes - table_bytes;
    int cur = 0;
    const ValT* vin = vals_first;
    const int passes = (key_bits + kRadixBits - 1) / kRadixBits;
    for (int p = 0; p < passes; ++p) {
        const int shift = p * kRadixBits;
        hipLaunchKernelGGL((k_radix_count<KeyT, ITEMS>), dim3((unsigned)tiles), dim3(kSortThreads), 0, s,
                           (const KeyT*)keys[cur], n, shift, table, tiles);
        const insum_status st = exclusive_scan_i32(scan_temp, scan_bytes, table, table, tiles * kRadix, s);
        if (st != INSUM_OK) return -(int)st;
        hipLaunchKernelGGL((k_radix_scatter<KeyT, ValT, ITEMS>), dim3((unsigned)tiles), dim3(kSortThreads), 0, s,
                           (const KeyT*)keys[cur], vin, keys[cur ^ 1], vals[cur ^ 1], n, shift,
                           (const int32_t*)table, tiles);
        cur ^= 1;
        vin = vals[cur];
    }
    if (hipGetLastError() != hipSuccess) return -(int)INSUM_ERR_HIP;
    if (passes == 0 && vals_first != vals[0]) {
        if (hipMemcpyAsync(vals[0], vals_first, (size_t)n * sizeof(ValT), hipMemcpyDeviceToDevice, s) != hipSuccess)
            return -(int)INSUM_ERR_HIP;
    }
    return cur;
}

}  // namespace insum
