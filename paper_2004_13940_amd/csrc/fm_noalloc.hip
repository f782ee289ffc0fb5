// fm_forward_noalloc: steps 1-3 of the pass for callers that cannot allocate device memory
// (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
//
// fm_forward keeps two scratch buffers in the handle's workspace: one (loss, multiplier) pair of
// floats per workgroup of the row kernel, and the stage-1 sums of the reduction over those pairs.
// Here both live in a file-scope device array of fixed size.  Every GPU the library runs on holds
// its own copy of the array at its own address until the process ends; the address is resolved
// once per device when a handle is created there.  Host code never uses the array's name as a
// pointer: only the resolved address is passed to kernels.
#include "fm_internal.h"

namespace {

constexpr int64_t NOALLOC_MAX_BLOCKS = 262144;  // workgroups of the row kernel (2 MiB of pairs)
constexpr size_t PAIR_BYTES = (size_t)NOALLOC_MAX_BLOCKS * 2 * sizeof(float);
constexpr size_t SCRATCH_BYTES = PAIR_BYTES + (size_t)FM_REDUCE_TMP * sizeof(double);

static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
unsigned char* g_scratch_ptr[MAX_DEVICES] = {nullptr};  // device address of `scratch` on each device

}  // namespace

int fm_noalloc_init_device(fm_matrix* m)
{
    int dev = -1;
    FM_HIP(m, hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fm_fail(m, FM_ERANGE, "device %d outside 0..%d", dev, MAX_DEVICES - 1);
    if (g_scratch_ptr[dev] != nullptr) return FM_OK;
    void* ptr = nullptr;
    FM_HIP(m, hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (ptr == nullptr) return fm_fail(m, FM_EHIP, "static scratch has no address on device %d", dev);
    g_scratch_ptr[dev] = static_cast<unsigned char*>(ptr);
    return FM_OK;
}

extern "C" int fm_forward_noalloc(fm_matrix* m, const fm_params* p, const float* y, const float* w0, const float* w,
                                  const float* V, float* yhat, float* a, float* G, float* q, float* r,
                                  double* sums, void* hip_stream)
{
    if (m == nullptr) return FM_EINVAL;
    if (p == nullptr) return fm_fail(m, FM_EINVAL, "params is NULL");
    int vec, lanes;
    if (!fm_shape_for_K(p->K, &vec, &lanes))
        return fm_fail(m, FM_EINVAL, "K=%d unsupported (1..64, or a multiple of 4 up to 256)", p->K);
    if (p->loss != FM_LOSS_SQUARED && p->loss != FM_LOSS_LOGISTIC) return fm_fail(m, FM_EINVAL, "unknown loss %d", p->loss);
    if (w0 == nullptr || w == nullptr || V == nullptr) return fm_fail(m, FM_EINVAL, "w0, w, V must not be NULL");
    if ((r != nullptr || sums != nullptr) && y == nullptr) return fm_fail(m, FM_EINVAL, "r and sums need y");
    FM_TRY(fm_check_vec_aligned(m, {V, G}));
    if (p->half_gather) return fm_fail(m, FM_EINVAL, "half_gather needs a buffer for the copy of V: use fm_forward");
    if (m->prof) return fm_fail(m, FM_ESTATE, "per-kernel timing creates events: switch it off for this call");
    int dev = -1;
    FM_HIP(m, hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES || g_scratch_ptr[dev] == nullptr)
        return fm_fail(m, FM_ESTATE, "no static scratch on the current device (the handle was created on another one)");
    const int64_t blocks = fm_rows_grid(m->N, p->K);
    if (sums != nullptr && blocks > NOALLOC_MAX_BLOCKS)
        return fm_fail(m, FM_ERANGE, "N=%lld at K=%d needs %lld workgroups; the static scratch holds the sums of %lld",
                       (long long)m->N, p->K, (long long)blocks, (long long)NOALLOC_MAX_BLOCKS);
    hipStream_t st = (hipStream_t)hip_stream;
    float* pairs = reinterpret_cast<float*>(g_scratch_ptr[dev]);
    double* tmp = reinterpret_cast<double*>(g_scratch_ptr[dev] + PAIR_BYTES);
    if (m->N == 0) {
        if (sums == nullptr) return FM_OK;
        // a reduction over zero pairs writes the two zeros (no memset: the caller may be capturing)
        return fm_reduce_pairs(m, pairs, 0, sums, st, tmp);
    }
    RowArgs A = {};
    A.N = m->N;
    A.K = p->K;
    A.rowptr = m->rowptr;
    A.col = m->col;
    A.val = m->val;
    A.w0 = w0;
    A.w = w;
    A.V = V;
    A.y = y;
    A.yhat = yhat;
    A.a = a;
    A.G = G;
    A.q = q;
    A.r = r;
    A.gs = p->K;
    A.ss = 1;
    // every workgroup of the launch writes its pair, and the reduction reads exactly those: nothing
    // in the scratch has to start at zero
    A.row_part = sums != nullptr ? pairs : nullptr;
    A.loss = p->loss;
    A.s = p->loss_scale;
    FM_TRY(fm_launch_rows(m, A, false, st));
    if (sums != nullptr) FM_TRY(fm_reduce_pairs(m, pairs, blocks, sums, st, tmp));
    return FM_OK;
}
