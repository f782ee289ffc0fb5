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

enum { MODE_FORWARD = 0, MODE_REFRESH = 1 };

template <int L>
struct Chunk {
    static constexpr int CH = (16 / L) > 0 ? (16 / L) : 1;  // entry slots per lane and iteration
};

// Loss value and multiplier for one example (cases after eq. updates_v; the loss
// constants make the printed multiplier the exact derivative).  expf only ever sees
// a non-positive argument.
__device__ __forceinline__ void loss_and_multiplier(int32_t loss, float s, float yh, float y, float& l, float& r)
{
    if (loss == FM_LOSS_SQUARED) {
        const float d = yh - y;
        l = 0.5f * d * d;
        r = s * d;
    } else {
        const float mg = y * yh;
        if (mg > 0.f) {
            const float e = expf(-mg);
            l = log1pf(e);
            r = -s * y * e / (1.f + e);
        } else {
            const float e = expf(mg);
            l = -mg + log1pf(e);
            r = -s * y / (1.f + e);
        }
    }
}

template <int VEC, int L, int MODE>
__global__ __launch_bounds__(FM_BLOCK) void k_rows(const RowArgs A)
{
    constexpr int R = FM_WAVE / L;  // rows per wavefront
    constexpr int CH = Chunk<L>::CH;
    const int lane = threadIdx.x & (FM_WAVE - 1);
    const int wave = threadIdx.x / FM_WAVE;
    const int sub = lane & (L - 1);
    const int grp = lane / L;
    const int64_t row = (int64_t)blockIdx.x * (FM_WAVES * R) + wave * R + grp;
    const bool valid = row < A.N;
    int64_t beg = 0, end = 0;
    if (valid) {
        beg = A.rowptr[row];
        end = A.rowptr[row + 1];
    }
    const int K = A.K;
    const int kbase = sub * VEC;
    const bool kact = kbase < K;  // K is a multiple of VEC, so the whole slice is in range

    float acc[VEC];
#pragma unroll
    for (int u = 0; u < VEC; ++u) acc[u] = 0.f;
    float a_acc = 0.f, q_acc = 0.f;

    for (int64_t e = beg; e < end; e += L * CH) {
        int c[CH];
        float x[CH];
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int64_t my = e + u * L + sub;
            const bool has = my < end;
            c[u] = has ? A.col[my] : 0;
            x[u] = has ? A.val[my] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            if (e + u * L + sub < end) {
                if constexpr (MODE == MODE_FORWARD) {
                    a_acc += A.w[c[u]] * x[u];
                } else {
                    const float2 d = A.dwn[c[u]];
                    a_acc += d.x * x[u];
                    q_acc += d.y * x[u] * x[u];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < CH; ++u) {
#pragma unroll
            for (int t = 0; t < L; ++t) {
                const int ct = fm_group_bcast<L>(c[u], t);
                const float xt = fm_group_bcast<L>(x[u], t);
                if (e + u * L + t < end && kact) {
                    float v[VEC];
                    fm_load_vec<VEC>(A.V + (int64_t)ct * K + kbase, v);
#pragma unroll
                    for (int z = 0; z < VEC; ++z) {
                        acc[z] += v[z] * xt;
                        if constexpr (MODE == MODE_FORWARD) q_acc += v[z] * v[z] * (xt * xt);
                    }
                }
            }
        }
    }

    float l_i = 0.f, r_i = 0.f;
    if constexpr (MODE == MODE_FORWARD) {
        float pair = 0.f;
#pragma unroll
        for (int z = 0; z < VEC; ++z) pair += acc[z] * acc[z];
        const float a_i = fm_group_sum<L>(a_acc);
        const float q_i = fm_group_sum<L>(q_acc);
        pair = fm_group_sum<L>(pair);
        const float yh = A.w0[0] + a_i + 0.5f * (pair - q_i);
        if (valid) {
            if (A.G != nullptr && kact) fm_store_vec<VEC>(A.G + row * K + kbase, acc);
            if (sub == 0) {
                if (A.a != nullptr) A.a[row] = a_i;
                if (A.q != nullptr) A.q[row] = q_i;
                if (A.yhat != nullptr) A.yhat[row] = yh;
                if (A.y != nullptr) {
                    loss_and_multiplier(A.loss, A.s, yh, A.y[row], l_i, r_i);
                    if (A.r != nullptr) A.r[row] = r_i;
                }
            }
        }
    } else {
        // rows that have no entry in this stratum keep their aggregates untouched
        const bool touched = valid && beg < end;  // uniform inside a group
        const float da = fm_group_sum<L>(a_acc);
        const float dq = fm_group_sum<L>(q_acc);
        float pair = 0.f;
        if (touched && kact) {
            float g[VEC];
            fm_load_vec<VEC>(A.G + row * K + kbase, g);
#pragma unroll
            for (int z = 0; z < VEC; ++z) {
                g[z] += acc[z];
                pair += g[z] * g[z];
            }
            fm_store_vec<VEC>(A.G + row * K + kbase, g);
        }
        pair = fm_group_sum<L>(pair);
        if (touched && sub == 0) {
            const float a_i = A.a[row] + da;
            const float q_i = A.q[row] + dq;
            A.a[row] = a_i;
            A.q[row] = q_i;
            const float yh = A.w0[0] + a_i + 0.5f * (pair - q_i);
            if (A.yhat != nullptr) A.yhat[row] = yh;
            loss_and_multiplier(A.loss, A.s, yh, A.y[row], l_i, r_i);
            A.r[row] = r_i;
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
    if (refresh)
        hipLaunchKernelGGL((k_rows<VEC, L, MODE_REFRESH>), dim3((unsigned)grid), dim3(FM_BLOCK), 0, st, A);
    else
        hipLaunchKernelGGL((k_rows<VEC, L, MODE_FORWARD>), dim3((unsigned)grid), dim3(FM_BLOCK), 0, st, A);
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
    int vec, lanes;
    if (!fm_shape_for_K(A.K, &vec, &lanes)) return fm_fail(m, FM_EINVAL, "unsupported K=%d", A.K);
    switch (vec) {
        case 4: return launch_rows_v<4>(m, lanes, A, refresh, st);
        case 2: return launch_rows_v<2>(m, lanes, A, refresh, st);
        default: return launch_rows_v<1>(m, lanes, A, refresh, st);
    }
}
