// Deterministic reductions (fixed order, fp64 accumulation) and the bias step.
#include "fm_device.h"
#include "fm_internal.h"

namespace {

constexpr int RED_THREADS = 1024;
constexpr int RED_BLOCKS = FM_REDUCE_TMP;

__device__ __forceinline__ double block_sum_1024(double v, double* sh)
{
    v = fm_wave_sum(v);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) sh[wave] = v;
    __syncthreads();
    double t = 0.0;
    if (threadIdx.x == 0)
        for (int i = 0; i < RED_THREADS / 64; ++i) t += sh[i];
    __syncthreads();
    return t;  // valid in thread 0
}

// part holds n interleaved pairs (x0,x1).  Stage 1: workgroup b sums its contiguous share of the
// pairs into tmp[2b], tmp[2b+1]; stage 2: one workgroup adds the nb partial pairs into out2.
__global__ __launch_bounds__(RED_THREADS) void k_reduce_pairs(const float* __restrict__ part, int64_t n,
                                                              double* __restrict__ tmp)
{
    __shared__ double sh[RED_THREADS / 64];
    const int64_t chunk = (n + gridDim.x - 1) / gridDim.x;
    const int64_t lo = (int64_t)blockIdx.x * chunk;
    const int64_t hi = lo + chunk < n ? lo + chunk : n;
    double s0 = 0.0, s1 = 0.0;
    const float2* p2 = reinterpret_cast<const float2*>(part);
    for (int64_t i = lo + threadIdx.x; i < hi; i += RED_THREADS) {
        const float2 v = p2[i];
        s0 += (double)v.x;
        s1 += (double)v.y;
    }
    const double t0 = block_sum_1024(s0, sh);
    const double t1 = block_sum_1024(s1, sh);
    if (threadIdx.x == 0) {
        tmp[2 * blockIdx.x] = t0;
        tmp[2 * blockIdx.x + 1] = t1;
    }
}

__global__ __launch_bounds__(RED_THREADS) void k_reduce_pairs_final(const double* __restrict__ tmp, int nb,
                                                                    double* __restrict__ out2)
{
    __shared__ double sh[RED_THREADS / 64];
    double s0 = 0.0, s1 = 0.0;
    for (int i = threadIdx.x; i < nb; i += RED_THREADS) {
        s0 += tmp[2 * i];
        s1 += tmp[2 * i + 1];
    }
    const double t0 = block_sum_1024(s0, sh);
    const double t1 = block_sum_1024(s1, sh);
    if (threadIdx.x == 0) {
        out2[0] = t0;
        out2[1] = t1;
    }
}

__global__ __launch_bounds__(RED_THREADS) void k_reduce_stage1(const float* __restrict__ x, int64_t n, int64_t stride,
                                                               int square, double* __restrict__ tmp)
{
    __shared__ double sh[RED_THREADS / 64];
    const int64_t chunk = (n + gridDim.x - 1) / gridDim.x;
    const int64_t lo = (int64_t)blockIdx.x * chunk;
    const int64_t hi = lo + chunk < n ? lo + chunk : n;
    double s = 0.0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += RED_THREADS) {
        const double v = (double)x[i * stride];
        s += square ? v * v : v;
    }
    const double t = block_sum_1024(s, sh);
    if (threadIdx.x == 0) tmp[blockIdx.x] = t;
}

__global__ __launch_bounds__(RED_THREADS) void k_reduce_stage2(const double* __restrict__ tmp, int nb,
                                                               double* __restrict__ out1)
{
    __shared__ double sh[RED_THREADS / 64];
    double s = 0.0;
    for (int i = threadIdx.x; i < nb; i += RED_THREADS) s += tmp[i];
    const double t = block_sum_1024(s, sh);
    if (threadIdx.x == 0) out1[0] = t;
}

// what = 0: sum of (yhat - y)^2 ; what = 1: number of i with sign(yhat_i) == y_i (0 counts as +1)
__global__ __launch_bounds__(RED_THREADS) void k_eval_stage1(const float* __restrict__ yhat,
                                                             const float* __restrict__ y, int64_t n, int what,
                                                             double* __restrict__ tmp)
{
    __shared__ double sh[RED_THREADS / 64];
    const int64_t chunk = (n + gridDim.x - 1) / gridDim.x;
    const int64_t lo = (int64_t)blockIdx.x * chunk;
    const int64_t hi = lo + chunk < n ? lo + chunk : n;
    double s = 0.0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += RED_THREADS) {
        const float f = yhat[i], t = y[i];
        if (what == 0) {
            const double d = (double)f - (double)t;
            s += d * d;
        } else {
            s += ((f >= 0.f ? 1.f : -1.f) == t) ? 1.0 : 0.0;
        }
    }
    const double tot = block_sum_1024(s, sh);
    if (threadIdx.x == 0) tmp[blockIdx.x] = tot;
}

__global__ void k_fill_i32(int32_t* __restrict__ x, int64_t n, int32_t v)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) x[i] = v;
}

__global__ void k_bias(float* w0, const double* rsum, float eta, float* grad_out)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        const float g = (float)rsum[0];
        if (grad_out != nullptr) grad_out[0] = g;
        if (w0 != nullptr) w0[0] = w0[0] - eta * g;
    }
}

}  // namespace

int fm_reduce_pairs(fm_matrix* m, const float* part, int64_t nblocks, double* out2, hipStream_t st, double* tmp)
{
    // stage-1 scratch of FM_REDUCE_TMP doubles (pairs: at most RED_BLOCKS / 2 workgroups); by default
    // scal[8..8+RED_BLOCKS)
    if (tmp == nullptr) tmp = m->scal + 8;
    int nb = (int)((nblocks + 4 * RED_THREADS - 1) / (4 * RED_THREADS));
    if (nb < 1) nb = 1;
    if (nb > RED_BLOCKS / 2) nb = RED_BLOCKS / 2;
    ProfScope ps(m, st, FMK_REDUCE);
    hipLaunchKernelGGL(k_reduce_pairs, dim3(nb), dim3(RED_THREADS), 0, st, part, nblocks, tmp);
    FM_HIP(m, hipGetLastError());
    hipLaunchKernelGGL(k_reduce_pairs_final, dim3(1), dim3(RED_THREADS), 0, st, (const double*)tmp, nb, out2);
    FM_HIP(m, hipGetLastError());
    return FM_OK;
}

int fm_reduce_sum(fm_matrix* m, const float* x, int64_t n, int64_t stride, bool square, double* out1, hipStream_t st)
{
    // scal[8..8+RED_BLOCKS) is the stage-1 scratch
    double* tmp = m->scal + 8;
    int nb = (int)((n + 16 * RED_THREADS - 1) / (16 * RED_THREADS));
    if (nb < 1) nb = 1;
    if (nb > RED_BLOCKS) nb = RED_BLOCKS;
    ProfScope ps(m, st, FMK_REDUCE);
    hipLaunchKernelGGL(k_reduce_stage1, dim3(nb), dim3(RED_THREADS), 0, st, x, n, stride, square ? 1 : 0, tmp);
    FM_HIP(m, hipGetLastError());
    hipLaunchKernelGGL(k_reduce_stage2, dim3(1), dim3(RED_THREADS), 0, st, (const double*)tmp, nb, out1);
    FM_HIP(m, hipGetLastError());
    return FM_OK;
}

int fm_reduce_eval(fm_matrix* m, const float* yhat, const float* y, int64_t n, int what, double* out1, hipStream_t st)
{
    double* tmp = m->scal + 8;
    int nb = (int)((n + 16 * RED_THREADS - 1) / (16 * RED_THREADS));
    if (nb < 1) nb = 1;
    if (nb > RED_BLOCKS) nb = RED_BLOCKS;
    ProfScope ps(m, st, FMK_REDUCE);
    hipLaunchKernelGGL(k_eval_stage1, dim3(nb), dim3(RED_THREADS), 0, st, yhat, y, n, what, tmp);
    FM_HIP(m, hipGetLastError());
    hipLaunchKernelGGL(k_reduce_stage2, dim3(1), dim3(RED_THREADS), 0, st, (const double*)tmp, nb, out1);
    FM_HIP(m, hipGetLastError());
    return FM_OK;
}

// A fill by a kernel (not a memset node), so that a caller may capture the epoch into a graph.
int fm_fill_i32(fm_matrix* m, int32_t* x, int64_t n, int32_t v, hipStream_t st)
{
    if (n <= 0) return FM_OK;
    const int64_t grid = (n + 255) / 256;
    if (grid > 0x7fffffffLL) return fm_fail(m, FM_ERANGE, "fill too large");
    hipLaunchKernelGGL(k_fill_i32, dim3((unsigned)grid), dim3(256), 0, st, x, n, v);
    FM_HIP(m, hipGetLastError());
    return FM_OK;
}

int fm_bias_step(fm_matrix* m, float* w0, const double* rsum, float eta, float* grad_w0_out, hipStream_t st)
{
    ProfScope ps(m, st, FMK_BIAS);
    hipLaunchKernelGGL(k_bias, dim3(1), dim3(64), 0, st, w0, rsum, eta, grad_w0_out);
    FM_HIP(m, hipGetLastError());
    return FM_OK;
}
