// Row-side kernels: the fused forward pass (aggregates, prediction, loss, multiplier)
// and the incremental refresh of the aggregates of a stratified step.
//
// Layout: a wavefront is split into groups of L lanes; one group owns one row, lane
// `sub` of the group owns VEC consecutive latent dimensions [sub*VEC, sub*VEC+VEC).
// A group reads its row's (column, value) pairs L*CH at a time (one entry per lane
// and slot, coalesced), broadcasts each pair inside the group and gathers the V row
// of that column as one contiguous 4*K-byte request.
#include "fm_device.h"
#include "fm_internal.h"

namespace {

enum { MODE_FORWARD = 0, MODE_REFRESH = 1, MODE_FORWARD_HALF = 2 };  // the last: V rows from the half-precision copy

template <int VEC, int L, int MODE>
__global__ __launch_bounds__(FM_BLOCK) void k_rows(const RowArgs A)
{
    constexpr int R = FM_WAVE / L;  // rows per wavefront
    const int lane = threadIdx.x & (FM_WAVE - 1);
    const int wave = threadIdx.x / FM_WAVE;
    const int sub = lane & (L - 1);
    const int grp = lane / L;
    const int64_t slot = (int64_t)blockIdx.x * (FM_WAVES * R) + wave * R + grp;
    const bool valid = slot < A.N;
    int64_t row = slot;
    int64_t beg = 0, end = 0;
    if (valid) {
        int64_t at = slot;
        if constexpr (MODE == MODE_REFRESH) {
            if (A.rows != nullptr)
                row = A.rows[slot];  // pointers are indexed by list position
            else
                at = row;
        }
        beg = A.rowptr[at];
        end = A.rowptr[at + 1];
    }
    const int K = A.K;
    const int kbase = sub * VEC;
    const bool kact = kbase < K;  // K is a multiple of VEC, so the whole slice is in range

    float acc[VEC];
#pragma unroll
    for (int u = 0; u < VEC; ++u) acc[u] = 0.f;
    float a_acc = 0.f, q_acc = 0.f;
    const int kb = kact ? kbase : 0;
    [[maybe_unused]] bool touched = false;
    [[maybe_unused]] float g_old[VEC] = {};
    [[maybe_unused]] float a_old = 0.f, q_old = 0.f;
    if constexpr (MODE == MODE_FORWARD) {
        const float* __restrict__ w = A.w;
        fm_gather_accumulate<VEC, L, true>(A.col, A.val, beg, end, A.V, K, sub, kb, acc, q_acc,
                                           [&](int c, float x) {
                                               a_acc += w[c] * x;
                                               return x;
                                           });
    } else if constexpr (MODE == MODE_FORWARD_HALF) {
        const float* __restrict__ w = A.w;
        fm_gather_accumulate<VEC, L, true>(A.col, A.val, beg, end, A.Vh, K, sub, kb, acc, q_acc,
                                           [&](int c, float x) {
                                               a_acc += w[c] * x;
                                               return x;
                                           });
    } else {
        // rows that have no entry in this stratum keep their aggregates untouched
        touched = valid && beg < end;  // uniform inside a group
        if (touched) {  // issued before the gathers so that it overlaps them
            if (kact) fm_load_vec<VEC>(A.G + row * A.gs + kbase, g_old);
            if (sub == 0) {
                a_old = A.a[row * A.ss];
                q_old = A.q[row * A.ss];
            }
        }
        const float2* __restrict__ dwn = A.dwn;
        float unused = 0.f;
        // a row has few entries inside one stratum: one slot of L entries at a time keeps the
        // register count low, so that more rows are in flight
        fm_gather_accumulate<VEC, L, false, 1>(A.col, A.val, beg, end, A.V, K, sub, kb, acc, unused,
                                            [&](int c, float x) {
                                                const float2 d = dwn[c];
                                                a_acc += d.x * x;
                                                q_acc += d.y * (x * x);
                                                return x;
                                            });
    }
    if (!kact) {  // idle lanes of a group wider than K/VEC worked on a valid but foreign slice
#pragma unroll
        for (int u = 0; u < VEC; ++u) acc[u] = 0.f;
        if constexpr (MODE != MODE_REFRESH) q_acc = 0.f;
    }

    float l_i = 0.f, r_i = 0.f;
    if constexpr (MODE != MODE_REFRESH) {
        float pair = 0.f;
#pragma unroll
        for (int z = 0; z < VEC; ++z) pair += acc[z] * acc[z];
        const float a_i = fm_group_sum<L>(a_acc);
        const float q_i = fm_group_sum<L>(q_acc);
        pair = fm_group_sum<L>(pair);
        const float yh = A.w0[0] + a_i + 0.5f * (pair - q_i);
        if (valid) {
            if (sub == 0) {
                if (A.yhat != nullptr) A.yhat[row] = yh;
                if (A.y != nullptr) loss_and_multiplier(A.loss, A.s, yh, A.y[row], l_i, r_i);
            }
            if (A.G != nullptr && kact) fm_store_vec<VEC>(A.G + row * A.gs + kbase, acc);
            if (A.whole_rows) {
                // packed aggregate rows: [r | a | q] and the padding behind G go out as float4 too, so
                // that every 128-byte line of the row is written whole
                if constexpr (VEC == 4) {
                    const int tail4 = (int)(A.gs - K) / 4;
                    for (int t = sub; t < tail4; t += L) {
                        float z[4] = {0.f, 0.f, 0.f, 0.f};
                        if (t == 0) {
                            z[0] = r_i;
                            z[1] = a_i;
                            z[2] = q_i;
                        }
                        fm_store_vec<4>(A.G + row * A.gs + K + 4 * t, z);
                    }
                }
            } else if (sub == 0) {
                if (A.a != nullptr) A.a[row * A.ss] = a_i;
                if (A.q != nullptr) A.q[row * A.ss] = q_i;
                if (A.y != nullptr && A.r != nullptr) A.r[row * A.ss] = r_i;
            }
        }
    } else {
        const float da = fm_group_sum<L>(a_acc);
        const float dq = fm_group_sum<L>(q_acc);
        float pair = 0.f;
        float g[VEC];
#pragma unroll
        for (int z = 0; z < VEC; ++z) {
            g[z] = g_old[z] + acc[z];
            pair += g[z] * g[z];
        }
        if (!(touched && kact)) pair = 0.f;
        pair = fm_group_sum<L>(pair);
        float a_i = 0.f, q_i = 0.f;
        if (touched && sub == 0) {
            a_i = a_old + da;
            q_i = q_old + dq;
            const float yh = A.w0[0] + a_i + 0.5f * (pair - q_i);
            if (A.yhat != nullptr) A.yhat[row] = yh;
            loss_and_multiplier(A.loss, A.s, yh, A.y[row], l_i, r_i);
        }
        // all stores of a row together, so that its line is written back once
        if (touched && kact) fm_store_vec<VEC>(A.G + row * A.gs + kbase, g);
        if (touched && sub == 0) {
            A.r[row * A.ss] = r_i;
            A.a[row * A.ss] = a_i;
            A.q[row * A.ss] = q_i;
        }
    }

    if (A.row_part != nullptr) {
        // l_i, r_i are non-zero only in lane 0 of a group: fixed-order block sums
        __shared__ float sh[2 * FM_WAVES];
        const float ls = fm_wave_sum(l_i);
        const float rs = fm_wave_sum(r_i);
        if (lane == 0) {
            sh[wave] = ls;
            sh[FM_WAVES + wave] = rs;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            float t0 = 0.f, t1 = 0.f;
#pragma unroll
            for (int wv = 0; wv < FM_WAVES; ++wv) {
                t0 += sh[wv];
                t1 += sh[FM_WAVES + wv];
            }
            A.row_part[2 * (int64_t)blockIdx.x] = t0;
            A.row_part[2 * (int64_t)blockIdx.x + 1] = t1;
        }
    }
}

template <int VEC, int L>
int launch_rows_t(fm_matrix* m, const RowArgs& A, bool refresh, hipStream_t st)
{
    constexpr int R = FM_WAVE / L;
    const int64_t grid = (A.N + FM_WAVES * R - 1) / (FM_WAVES * R);
    if (grid <= 0) return FM_OK;
    if (grid > 0x7fffffffLL) return fm_fail(m, FM_ERANGE, "row grid too large");
    ProfScope ps(m, st, refresh ? FMK_ROWS_REFRESH : FMK_ROWS_FORWARD);
    if (refresh) {
        hipLaunchKernelGGL((k_rows<VEC, L, MODE_REFRESH>), dim3((unsigned)grid), dim3(FM_BLOCK), 0, st, A);
    } else if (A.Vh != nullptr) {
        if constexpr (VEC == 4)
            hipLaunchKernelGGL((k_rows<VEC, L, MODE_FORWARD_HALF>), dim3((unsigned)grid), dim3(FM_BLOCK), 0, st, A);
        else
            return fm_fail(m, FM_EINVAL, "half_gather needs K to be a multiple of 4");
    } else {
        hipLaunchKernelGGL((k_rows<VEC, L, MODE_FORWARD>), dim3((unsigned)grid), dim3(FM_BLOCK), 0, st, A);
    }
    FM_HIP(m, hipGetLastError());
    return FM_OK;
}

template <int VEC>
int launch_rows_v(fm_matrix* m, int lanes, const RowArgs& A, bool refresh, hipStream_t st)
{
    switch (lanes) {
        case 1: return launch_rows_t<VEC, 1>(m, A, refresh, st);
        case 2: return launch_rows_t<VEC, 2>(m, A, refresh, st);
        case 4: return launch_rows_t<VEC, 4>(m, A, refresh, st);
        case 8: return launch_rows_t<VEC, 8>(m, A, refresh, st);
        case 16: return launch_rows_t<VEC, 16>(m, A, refresh, st);
        case 32: return launch_rows_t<VEC, 32>(m, A, refresh, st);
        case 64: return launch_rows_t<VEC, 64>(m, A, refresh, st);
    }
    return fm_fail(m, FM_EINVAL, "unsupported lane count %d", lanes);
}

}  // namespace

namespace {
__global__ void k_unpack_aux(const FmAux x, int64_t N, int32_t K, float* a, float* G, float* q, float* r)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t per = K + 3;
    if (t >= N * per) return;
    const int64_t i = t / per;
    const int c = (int)(t % per);
    if (c < K) {
        if (G != nullptr) G[i * K + c] = x.G[i * x.gs + c];
    } else if (c == K) {
        if (r != nullptr) r[i] = x.r[i * x.ss];
    } else if (c == K + 1) {
        if (a != nullptr) a[i] = x.a[i * x.ss];
    } else {
        if (q != nullptr) q[i] = x.q[i * x.ss];
    }
}
}  // namespace

namespace {
// Caller-side dense r[N], G[N x K] into the packed aggregate rows [G | r | 0 | 0 | pad], one float4
// per thread, whole rows written.
__global__ void k_pack_aux(const FmAux x, int64_t N, int32_t K, const float* __restrict__ r,
                           const float* __restrict__ G)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t per = x.gs / 4;  // float4 per row
    if (t >= N * per) return;
    const int64_t i = t / per;
    const int o = (int)(t % per) * 4;
    float z[4] = {0.f, 0.f, 0.f, 0.f};
    if (o < K)
        fm_load_vec<4>(G + i * K + o, z);
    else if (o == K)
        z[0] = r[i];
    fm_store_vec<4>(x.G + i * x.gs + o, z);
}
}  // namespace

namespace {
__global__ void k_to_half(const float4* __restrict__ x, fm_h4* __restrict__ out, int64_t n4)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n4) return;
    const float4 v = x[i];
    fm_h4 h;
    h.x = (_Float16)v.x;
    h.y = (_Float16)v.y;
    h.z = (_Float16)v.z;
    h.w = (_Float16)v.w;
    out[i] = h;
}
}  // namespace

// n a multiple of 4; conversion rounds to nearest even (subnormal halves kept)
int fm_to_half(fm_matrix* m, const float* x, _Float16* out, int64_t n, hipStream_t st)
{
    const int64_t n4 = n / 4;
    if (n4 <= 0) return FM_OK;
    const int64_t grid = (n4 + 255) / 256;
    if (grid > 0x7fffffffLL) return fm_fail(m, FM_ERANGE, "conversion too large");
    hipLaunchKernelGGL(k_to_half, dim3((unsigned)grid), dim3(256), 0, st, reinterpret_cast<const float4*>(x),
                       reinterpret_cast<fm_h4*>(out), n4);
    FM_HIP(m, hipGetLastError());
    return FM_OK;
}

int fm_pack_aux(fm_matrix* m, const float* r, const float* G, hipStream_t st)
{
    const FmAux x = fm_aux_layout(m, m->wsK);
    const int64_t total = m->N * (x.gs / 4);
    if (total <= 0) return FM_OK;
    const int64_t grid = (total + 255) / 256;
    if (grid > 0x7fffffffLL) return fm_fail(m, FM_ERANGE, "aggregate copy too large");
    hipLaunchKernelGGL(k_pack_aux, dim3((unsigned)grid), dim3(256), 0, st, x, m->N, m->wsK, r, G);
    FM_HIP(m, hipGetLastError());
    return FM_OK;
}

int fm_unpack_aux(fm_matrix* m, float* a, float* G, float* q, float* r, hipStream_t st)
{
    const int64_t total = m->N * (int64_t)(m->wsK + 3);
    if (total <= 0) return FM_OK;
    const int64_t grid = (total + 255) / 256;
    if (grid > 0x7fffffffLL) return fm_fail(m, FM_ERANGE, "aggregate copy too large");
    hipLaunchKernelGGL(k_unpack_aux, dim3((unsigned)grid), dim3(256), 0, st, fm_aux_layout(m, m->wsK), m->N, m->wsK, a, G,
                       q, r);
    FM_HIP(m, hipGetLastError());
    return FM_OK;
}

bool fm_shape_for_K(int32_t K, int* vec, int* lanes)
{
    if (K < 1) return false;
    const int v = (K % 4 == 0) ? 4 : (K % 2 == 0) ? 2 : 1;
    int need = K / v, l = 1;
    while (l < need) l <<= 1;
    if (l > 64) return false;
    if (!(K <= 64 || (K % 4 == 0 && K <= 256))) return false;
    *vec = v;
    *lanes = l;
    return true;
}

int64_t fm_rows_grid(int64_t N, int32_t K)
{
    int vec, lanes;
    if (!fm_shape_for_K(K, &vec, &lanes)) return 0;
    const int64_t per = (int64_t)FM_WAVES * (FM_WAVE / lanes);
    return (N + per - 1) / per;
}

int fm_launch_rows(fm_matrix* m, const RowArgs& A, bool refresh, hipStream_t st)
{
    if (!refresh && A.dense_D > 0 && A.Vh == nullptr) return fm_launch_rows_dense(m, A, st);
    int vec, lanes;
    if (!fm_shape_for_K(A.K, &vec, &lanes)) return fm_fail(m, FM_EINVAL, "unsupported K=%d", A.K);
    switch (vec) {
        case 4: return launch_rows_v<4>(m, lanes, A, refresh, st);
        case 2: return launch_rows_v<2>(m, lanes, A, refresh, st);
        default: return launch_rows_v<1>(m, lanes, A, refresh, st);
    }
}
