// Calibration probes for the benchmark, built into a library of their own (libfm_bench_probe.so):
// not part of the method and not part of the product library.
//   bench_probe_gather  random rows of 64 or 128 bytes read per second from a buffer of a given size.
//                       The pass kernels are bound by this kind of traffic (gathers of V rows and of
//                       aggregate rows), so the figure is the ceiling their request rates are compared with.
//   bench_probe_copy    a plain device copy of known size, the reference the byte counters of the
//                       profiler are scaled by.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__device__ __forceinline__ uint32_t mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

// L lanes per row of L float4; every group reads `per` pseudo-random rows, 16 loads in flight.
template <int L>
__global__ __launch_bounds__(256) void k_probe_gather(const float4* __restrict__ buf, uint32_t nrows, int per,
                                                      float* __restrict__ sink)
{
    const int64_t gid = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / L;
    const int sub = threadIdx.x % L;
    float acc = 0.f;
    for (int it = 0; it < per; it += 16) {
        float4 v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const uint32_t r = mix32((uint32_t)(gid * 7919 + it + u)) % nrows;
            v[u] = buf[(int64_t)r * L + sub];
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) acc += v[u].x + v[u].w;
    }
    if (acc == 12345.678f) sink[0] = acc;  // never true for a zeroed buffer; keeps the loads
}

}  // namespace

extern "C" int bench_probe_gather(int64_t buffer_bytes, int32_t row_bytes, double* rows_per_s, void* hip_stream)
{
    if (rows_per_s == nullptr || (row_bytes != 64 && row_bytes != 128)) return -1;
    if (buffer_bytes < (1 << 20) || buffer_bytes > (int64_t(64) << 30)) return -1;
    hipStream_t st = (hipStream_t)hip_stream;
    const int L = row_bytes / 16;
    const int64_t nrows64 = buffer_bytes / row_bytes;
    if (nrows64 > 0xffffffffLL) return -4;
    void* buf = nullptr;
    float* sink = nullptr;
    hipEvent_t a = nullptr, b = nullptr;
    int rc = 0;
    if (hipMalloc(&buf, (size_t)nrows64 * row_bytes) != hipSuccess || hipMalloc((void**)&sink, 4) != hipSuccess) {
        (void)hipGetLastError();
        rc = -2;
    }
    if (rc == 0 && (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess)) rc = -6;
    if (rc == 0 && hipMemsetAsync(buf, 0, (size_t)nrows64 * row_bytes, st) != hipSuccess) rc = -6;
    const int per = 64;
    const int64_t groups = int64_t(4) << 20;  // 2.7e8 row reads per launch
    const unsigned grid = (unsigned)(groups * L / 256);
    float ms = 0.f;
    for (int rep = 0; rc == 0 && rep < 3; ++rep) {  // the last repetition is the one reported
        if (hipEventRecord(a, st) != hipSuccess) rc = -6;
        if (L == 4)
            hipLaunchKernelGGL(k_probe_gather<4>, dim3(grid), dim3(256), 0, st, (const float4*)buf, (uint32_t)nrows64, per, sink);
        else
            hipLaunchKernelGGL(k_probe_gather<8>, dim3(grid), dim3(256), 0, st, (const float4*)buf, (uint32_t)nrows64, per, sink);
        if (hipGetLastError() != hipSuccess || hipEventRecord(b, st) != hipSuccess || hipEventSynchronize(b) != hipSuccess ||
            hipEventElapsedTime(&ms, a, b) != hipSuccess)
            rc = -6;
    }
    if (rc == 0) *rows_per_s = ms > 0.f ? (double)groups * per / ((double)ms * 1e-3) : 0.0;
    if (a) (void)hipEventDestroy(a);
    if (b) (void)hipEventDestroy(b);
    if (buf) (void)hipFree(buf);
    if (sink) (void)hipFree(sink);
    return rc;
}

namespace {
__global__ __launch_bounds__(256) void k_probe_copy(const float4* __restrict__ src, float4* __restrict__ dst, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}
}  // namespace

// Copies `bytes` (a multiple of 16) from src to dst `reps` times with a plain kernel; both DEVICE, caller-owned.
extern "C" int bench_probe_copy(const void* src, void* dst, int64_t bytes, int32_t reps, void* hip_stream)
{
    if (src == nullptr || dst == nullptr || bytes <= 0 || bytes % 16 != 0 || reps < 1) return -1;
    const int64_t n = bytes / 16;
    const int64_t grid = (n + 255) / 256;
    if (grid > 0x7fffffffLL) return -4;
    for (int r = 0; r < reps; ++r)
        hipLaunchKernelGGL(k_probe_copy, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)hip_stream,
                           (const float4*)src, (float4*)dst, n);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}
