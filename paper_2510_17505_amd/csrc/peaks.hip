// Achievable-peak microbenchmarks for gfx950 (measurement tools, not part of the SpMM path;
// built into their own library, libinsum_peaks.so).  Each entry point allocates what it
// needs, times its kernel with HIP events and returns the rate; a negative value is an error.
//
//   insum_peak_copy_gbs         streaming copy, 4 x 16 bytes per lane in flight, non-temporal
//                                                                          -> GB/s (read + write)
//   insum_peak_read_gbs         streaming read of the same buffer (sum)    -> GB/s
//   insum_peak_random_read_gbs  every wavefront reads 1 KiB pieces at random 1 KiB-aligned
//                               offsets inside a working set               -> GB/s
//   insum_peak_random_rows_gbs  the same with pieces of 64 ... 1024 bytes read by 4 ... 64 lanes
//                               (the access pattern of a row gather)       -> GB/s
//   insum_peak_gather_store_gbs the same row reads with one row written per `gathers_per_store`
//                               reads, every lane group writing its own consecutive rows (the
//                               read/write mix of an SpMM whose rows hold that many entries)
//                                                                          -> GB/s (read + write)
//   insum_peak_mfma_tflops      register-resident v_mfma_f32_32x32x16_bf16 -> TFLOP/s
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// n is a multiple of 4 * 256 * gridDim.x (the callers round the size down).
__global__ __launch_bounds__(256) void k_copy(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += 4 * stride) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(v[u], dst + i + u * stride);
    }
}

__global__ __launch_bounds__(256) void k_read(const u32x4* __restrict__ src, size_t n, uint32_t* sink) {
    const size_t stride = (size_t)gridDim.x * 256;
    u32x4 acc = {0, 0, 0, 0};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += 8 * stride) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u];
    }
    if (acc.x == 0x12345678u) sink[0] = acc.y + acc.z + acc.w;  // keeps the loads alive
}

__global__ __launch_bounds__(256) void k_random_read(const char* __restrict__ src, size_t ws_kib, int iters, uint32_t* sink) {
    const int lane = threadIdx.x % 64;
    uint32_t state = (blockIdx.x * 4 + threadIdx.x / 64) * 2654435761u + 12345u;
    u32x4 acc = {0, 0, 0, 0};
    for (int i = 0; i < iters; i += 8) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            state = state * 1664525u + 1013904223u;  // same sequence in every lane of the wavefront
            v[u] = *reinterpret_cast<const u32x4*>(src + ((size_t)(state >> 8) % ws_kib) * 1024 + lane * 16);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u];
    }
    if (acc.x == 0x12345678u) sink[0] = acc.y + acc.z + acc.w;  // keeps the loads alive
}

// LPR lanes read one piece of LPR * 16 bytes; every group of LPR lanes follows its own sequence.
template <int LPR>
__global__ __launch_bounds__(256) void k_random_rows(const char* __restrict__ src, size_t pieces, int iters, uint32_t* sink) {
    const int sub = threadIdx.x % LPR;
    uint32_t state = (uint32_t)(((size_t)blockIdx.x * 256 + threadIdx.x) / LPR) * 2654435761u + 12345u;
    u32x4 acc = {0, 0, 0, 0};
    for (int i = 0; i < iters; i += 8) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            state = state * 1664525u + 1013904223u;
            v[u] = *reinterpret_cast<const u32x4*>(src + ((size_t)(state >> 4) % pieces) * (LPR * 16) + sub * 16);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u];
    }
    if (acc.x == 0x12345678u) sink[0] = acc.y + acc.z + acc.w;
}

// As k_random_rows, and after every `gps` reads (a multiple of 8) the group stores the running sum
// as one more row of its own output range [group * (iters / gps), ...) of dst.
template <int LPR>
__global__ __launch_bounds__(256) void k_gather_store(const char* __restrict__ src, size_t pieces, int iters, int gps,
                                                      char* __restrict__ dst, uint32_t* sink) {
    const int sub = threadIdx.x % LPR;
    const size_t group = ((size_t)blockIdx.x * 256 + threadIdx.x) / LPR;
    uint32_t state = (uint32_t)group * 2654435761u + 12345u;
    u32x4 acc = {0, 0, 0, 0};
    char* out = dst + group * (size_t)(iters / gps) * (LPR * 16) + sub * 16;
    int since = 0;
    for (int i = 0; i < iters; i += 8) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            state = state * 1664525u + 1013904223u;
            v[u] = *reinterpret_cast<const u32x4*>(src + ((size_t)(state >> 4) % pieces) * (LPR * 16) + sub * 16);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u];
        since += 8;
        if (since >= gps) {
            since = 0;
            __builtin_nontemporal_store(acc, reinterpret_cast<u32x4*>(out));
            out += LPR * 16;
        }
    }
    if (acc.x == 0x12345678u) sink[0] = acc.y + acc.z + acc.w;
}

__global__ __launch_bounds__(256) void k_mfma(int iters, float* sink) {
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(float)(threadIdx.x % 3);
        b[i] = (__bf16)(float)(threadIdx.x % 5);
    }
    f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
    const float s = c0[0] + c1[1] + c2[2] + c3[3];
    if (s == 12345.678f) sink[0] = s;
}

struct Timer {
    hipEvent_t e0, e1;
    bool ok;
    Timer() { ok = hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess; }
    ~Timer() {
        (void)hipEventDestroy(e0);
        (void)hipEventDestroy(e1);
    }
};

}  // namespace

extern "C" double insum_peak_copy_gbs(size_t bytes, int repeats) {
    Timer t;
    char *src = nullptr, *dst = nullptr;
    if (!t.ok || hipMalloc(&src, bytes) != hipSuccess || hipMalloc(&dst, bytes) != hipSuccess) return -1.0;
    (void)hipMemset(src, 1, bytes);
    const unsigned blocks = 256 * 16;
    const size_t n = bytes / 16 / (4 * 256 * blocks) * (4 * 256 * blocks);
    double best = -1.0;
    for (int r = 0; r < repeats + 1; ++r) {
        (void)hipEventRecord(t.e0);
        hipLaunchKernelGGL(k_copy, dim3(blocks), dim3(256), 0, 0, (const u32x4*)src, (u32x4*)dst, n);
        (void)hipEventRecord(t.e1);
        if (hipEventSynchronize(t.e1) != hipSuccess) { best = -1.0; break; }
        float ms = 0;
        (void)hipEventElapsedTime(&ms, t.e0, t.e1);
        if (r > 0 && 2.0 * n * 16 / ms / 1e6 > best) best = 2.0 * n * 16 / ms / 1e6;
    }
    (void)hipFree(src);
    (void)hipFree(dst);
    return best;
}

extern "C" double insum_peak_read_gbs(size_t bytes, int repeats) {
    Timer t;
    char* src = nullptr;
    uint32_t* sink = nullptr;
    if (!t.ok || hipMalloc(&src, bytes) != hipSuccess || hipMalloc(&sink, 4) != hipSuccess) return -1.0;
    (void)hipMemset(src, 1, bytes);
    const unsigned blocks = 256 * 16;
    const size_t n = bytes / 16 / (8 * 256 * blocks) * (8 * 256 * blocks);
    double best = -1.0;
    for (int r = 0; r < repeats + 1; ++r) {
        (void)hipEventRecord(t.e0);
        hipLaunchKernelGGL(k_read, dim3(blocks), dim3(256), 0, 0, (const u32x4*)src, n, sink);
        (void)hipEventRecord(t.e1);
        if (hipEventSynchronize(t.e1) != hipSuccess) { best = -1.0; break; }
        float ms = 0;
        (void)hipEventElapsedTime(&ms, t.e0, t.e1);
        if (r > 0 && (double)n * 16 / ms / 1e6 > best) best = (double)n * 16 / ms / 1e6;
    }
    (void)hipFree(src);
    (void)hipFree(sink);
    return best;
}

extern "C" double insum_peak_random_read_gbs(size_t working_set_bytes, int repeats) {
    Timer t;
    char* src = nullptr;
    uint32_t* sink = nullptr;
    if (working_set_bytes < (1 << 20)) working_set_bytes = 1 << 20;
    if (!t.ok || hipMalloc(&src, working_set_bytes) != hipSuccess || hipMalloc(&sink, 4) != hipSuccess) return -1.0;
    (void)hipMemset(src, 1, working_set_bytes);
    const int blocks = 256 * 8, iters = 512;
    double best = -1.0;
    for (int r = 0; r < repeats + 1; ++r) {
        (void)hipEventRecord(t.e0);
        hipLaunchKernelGGL(k_random_read, dim3(blocks), dim3(256), 0, 0, (const char*)src, working_set_bytes / 1024, iters, sink);
        (void)hipEventRecord(t.e1);
        if (hipEventSynchronize(t.e1) != hipSuccess) { best = -1.0; break; }
        float ms = 0;
        (void)hipEventElapsedTime(&ms, t.e0, t.e1);
        const double gbs = (double)blocks * 4 * iters * 1024 / ms / 1e6;
        if (r > 0 && gbs > best) best = gbs;
    }
    (void)hipFree(src);
    (void)hipFree(sink);
    return best;
}

extern "C" double insum_peak_random_rows_gbs(size_t working_set_bytes, int row_bytes, int repeats) {
    Timer t;
    char* src = nullptr;
    uint32_t* sink = nullptr;
    if (working_set_bytes < (1 << 20)) working_set_bytes = 1 << 20;
    if (row_bytes != 64 && row_bytes != 128 && row_bytes != 256 && row_bytes != 512 && row_bytes != 1024) return -1.0;
    if (!t.ok || hipMalloc(&src, working_set_bytes) != hipSuccess || hipMalloc(&sink, 4) != hipSuccess) return -1.0;
    (void)hipMemset(src, 1, working_set_bytes);
    const int blocks = 256 * 8, iters = 512;
    const size_t pieces = working_set_bytes / row_bytes;
    double best = -1.0;
    for (int r = 0; r < repeats + 1; ++r) {
        (void)hipEventRecord(t.e0);
        switch (row_bytes) {
            case 64: hipLaunchKernelGGL(k_random_rows<4>, dim3(blocks), dim3(256), 0, 0, (const char*)src, pieces, iters, sink); break;
            case 128: hipLaunchKernelGGL(k_random_rows<8>, dim3(blocks), dim3(256), 0, 0, (const char*)src, pieces, iters, sink); break;
            case 256: hipLaunchKernelGGL(k_random_rows<16>, dim3(blocks), dim3(256), 0, 0, (const char*)src, pieces, iters, sink); break;
            case 512: hipLaunchKernelGGL(k_random_rows<32>, dim3(blocks), dim3(256), 0, 0, (const char*)src, pieces, iters, sink); break;
            default: hipLaunchKernelGGL(k_random_rows<64>, dim3(blocks), dim3(256), 0, 0, (const char*)src, pieces, iters, sink); break;
        }
        (void)hipEventRecord(t.e1);
        if (hipEventSynchronize(t.e1) != hipSuccess) { best = -1.0; break; }
        float ms = 0;
        (void)hipEventElapsedTime(&ms, t.e0, t.e1);
        const double gbs = (double)blocks * 256 * iters * 16 / ms / 1e6;
        if (r > 0 && gbs > best) best = gbs;
    }
    (void)hipFree(src);
    (void)hipFree(sink);
    return best;
}

extern "C" double insum_peak_gather_store_gbs(size_t working_set_bytes, int row_bytes, int gathers_per_store,
                                              int repeats) {
    Timer t;
    char *src = nullptr, *dst = nullptr;
    uint32_t* sink = nullptr;
    if (working_set_bytes < (1 << 20)) working_set_bytes = 1 << 20;
    if (row_bytes != 256 && row_bytes != 512) return -1.0;
    const int blocks = 256 * 8, iters = 512;
    const int gps = gathers_per_store < 8 ? 8 : gathers_per_store > iters ? iters : gathers_per_store / 8 * 8;
    const size_t groups = (size_t)blocks * 256 / (row_bytes / 16);
    const size_t out_bytes = groups * (size_t)(iters / gps) * row_bytes;   // rows written per launch
    if (!t.ok || hipMalloc(&src, working_set_bytes) != hipSuccess || hipMalloc(&dst, out_bytes) != hipSuccess ||
        hipMalloc(&sink, 4) != hipSuccess) {
        (void)hipFree(src);
        (void)hipFree(dst);
        return -1.0;
    }
    (void)hipMemset(src, 1, working_set_bytes);
    const size_t pieces = working_set_bytes / row_bytes;
    double best = -1.0;
    for (int r = 0; r < repeats + 1; ++r) {
        (void)hipEventRecord(t.e0);
        if (row_bytes == 256)
            hipLaunchKernelGGL(k_gather_store<16>, dim3(blocks), dim3(256), 0, 0, (const char*)src, pieces, iters, gps, dst, sink);
        else
            hipLaunchKernelGGL(k_gather_store<32>, dim3(blocks), dim3(256), 0, 0, (const char*)src, pieces, iters, gps, dst, sink);
        (void)hipEventRecord(t.e1);
        if (hipEventSynchronize(t.e1) != hipSuccess) { best = -1.0; break; }
        float ms = 0;
        (void)hipEventElapsedTime(&ms, t.e0, t.e1);
        const double gbs = ((double)blocks * 256 * iters * 16 + (double)out_bytes) / ms / 1e6;
        if (r > 0 && gbs > best) best = gbs;
    }
    (void)hipFree(src);
    (void)hipFree(dst);
    (void)hipFree(sink);
    return best;
}

extern "C" double insum_peak_mfma_tflops(int repeats) {
    Timer t;
    float* sink = nullptr;
    if (!t.ok || hipMalloc(&sink, 4) != hipSuccess) return -1.0;
    const int blocks = 256 * 8, iters = 4096;
    double best = -1.0;
    for (int r = 0; r < repeats + 1; ++r) {
        (void)hipEventRecord(t.e0);
        hipLaunchKernelGGL(k_mfma, dim3(blocks), dim3(256), 0, 0, iters, sink);
        (void)hipEventRecord(t.e1);
        if (hipEventSynchronize(t.e1) != hipSuccess) { best = -1.0; break; }
        float ms = 0;
        (void)hipEventElapsedTime(&ms, t.e0, t.e1);
        const double tf = (double)blocks * 4 * iters * 4 * (2.0 * 32 * 32 * 16) / ms / 1e9;
        if (r > 0 && tf > best) best = tf;
    }
    (void)hipFree(sink);
    return best;
}
