// Column-side kernels: the atomic-free transposed product for the gradient
// (eqs. updates_w, updates_v) over a CSC copy, with the parameter step fused in.
//
//   gw_j   = sum_i x_ij r_i
//   s2_j   = sum_i x_ij^2 r_i
//   gV_jk  = sum_i x_ij r_i G_ik
//   grad_w_j  = gw_j + rho lambda_w w_j
//   grad_V_jk = gV_jk - s2_j v_jk + rho lambda_v v_jk
//
// A group of L lanes owns one column (lane `sub` holds VEC latent dimensions).
// Columns longer than FM_SEG entries are cut into fixed segments: k_cols skips them,
// k_cols_long writes one partial per segment and k_cols_finish adds the partials of a
// column in a fixed order, so results are bit-reproducible from run to run.
#include "fm_device.h"
#include "fm_internal.h"

namespace {

template <int L>
struct Chunk {
    static constexpr int CH = (16 / L) > 0 ? (16 / L) : 1;
};

// Accumulate one run of entries [beg,end) of a column into acc/gw/s2 (per-lane
// partials for gw, s2; complete sums for acc's latent slice).
template <int VEC, int L>
__device__ __forceinline__ void accumulate_entries(const ColArgs& A, int64_t beg, int64_t end, int sub, int kbase,
                                                   bool kact, float (&acc)[VEC], float& gw, float& s2)
{
    constexpr int CH = Chunk<L>::CH;
    const int K = A.K;
    for (int64_t e = beg; e < end; e += L * CH) {
        int ir[CH];
        float xr[CH];
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int64_t my = e + u * L + sub;
            const bool has = my < end;
            ir[u] = has ? A.row[my] : 0;
            const float x = has ? A.val[my] : 0.f;
            const float ri = has ? A.r[ir[u]] : 0.f;
            xr[u] = x * ri;
            gw += xr[u];
            s2 += x * xr[u];
        }
#pragma unroll
        for (int u = 0; u < CH; ++u) {
#pragma unroll
            for (int t = 0; t < L; ++t) {
                const int it = fm_group_bcast<L>(ir[u], t);
                const float xrt = fm_group_bcast<L>(xr[u], t);
                if (e + u * L + t < end && kact) {
                    float g[VEC];
                    fm_load_vec<VEC>(A.G + (int64_t)it * K + kbase, g);
#pragma unroll
                    for (int z = 0; z < VEC; ++z) acc[z] += xrt * g[z];
                }
            }
        }
    }
}

__device__ __forceinline__ float reg_share(const ColArgs& A, int64_t j)
{
    if (A.rb == nullptr) return 1.f;
    const int32_t qb = fm_block_of(j, A.D, A.P);
    int32_t p = (qb - A.s) % A.P;
    if (p < 0) p += A.P;
    return (float)((double)(A.rb[p + 1] - A.rb[p]) / (double)A.N);
}

// Turn the data sums of column j into the gradient, and either store it or take the
// step (optionally recording the change for the incremental refresh).
template <int VEC, int L, bool UPDATE>
__device__ __forceinline__ void finish_column(const ColArgs& A, int64_t j, int sub, int kbase, bool kact,
                                              const float (&acc)[VEC], float gw, float s2)
{
    const int K = A.K;
    const float rho = reg_share(A, j);
    float dn = 0.f;
    if (kact) {
        float v[VEC], g[VEC];
        fm_load_vec<VEC>(A.V + j * K + kbase, v);
#pragma unroll
        for (int z = 0; z < VEC; ++z) g[z] = acc[z] - s2 * v[z] + rho * A.lambda_v * v[z];
        if constexpr (UPDATE) {
            float d[VEC], vn[VEC];
#pragma unroll
            for (int z = 0; z < VEC; ++z) {
                d[z] = -A.eta * g[z];
                vn[z] = v[z] + d[z];
                dn += d[z] * (2.f * v[z] + d[z]);  // |v+d|^2 - |v|^2 without cancellation
            }
            fm_store_vec<VEC>(A.V + j * K + kbase, vn);
            if (A.dV != nullptr) fm_store_vec<VEC>(A.dV + j * K + kbase, d);
        } else {
            if (A.grad_V != nullptr) fm_store_vec<VEC>(A.grad_V + j * K + kbase, g);
        }
    }
    if constexpr (UPDATE) {
        if (A.dwn != nullptr) dn = fm_group_sum<L>(dn);
    }
    if (sub == 0) {
        const float wj = A.w[j];
        const float g = gw + rho * A.lambda_w * wj;
        if constexpr (UPDATE) {
            const float d = -A.eta * g;
            A.w[j] = wj + d;
            if (A.dwn != nullptr) A.dwn[j] = make_float2(d, dn);
        } else {
            if (A.grad_w != nullptr) A.grad_w[j] = g;
        }
    }
}

// All columns; those longer than FM_SEG entries are left to the two kernels below.
template <int VEC, int L, bool UPDATE>
__global__ __launch_bounds__(FM_BLOCK) void k_cols(const ColArgs A)
{
    constexpr int R = FM_WAVE / L;
    const int lane = threadIdx.x & (FM_WAVE - 1);
    const int wave = threadIdx.x / FM_WAVE;
    const int sub = lane & (L - 1);
    const int grp = lane / L;
    const int64_t j = (int64_t)blockIdx.x * (FM_WAVES * R) + wave * R + grp;
    const bool valid = j < A.D;
    int64_t beg = 0, end = 0;
    if (valid) {
        beg = A.ptr[j];
        end = A.ptr[j + 1];
    }
    const bool is_long = (end - beg) > FM_SEG;
    if (is_long) end = beg;
    const int kbase = sub * VEC;
    const bool kact = kbase < A.K;

    float acc[VEC];
#pragma unroll
    for (int z = 0; z < VEC; ++z) acc[z] = 0.f;
    float gw = 0.f, s2 = 0.f;
    accumulate_entries<VEC, L>(A, beg, end, sub, kbase, kact, acc, gw, s2);
    gw = fm_group_sum<L>(gw);
    s2 = fm_group_sum<L>(s2);

    float wsq = 0.f, vsq = 0.f;
    if (A.col_part != nullptr && valid) {  // |w|^2, |V|^2 at the parameters before the step
        if (kact) {
            float v[VEC];
            fm_load_vec<VEC>(A.V + j * A.K + kbase, v);
#pragma unroll
            for (int z = 0; z < VEC; ++z) vsq += v[z] * v[z];
        }
        if (sub == 0) {
            const float wj = A.w[j];
            wsq = wj * wj;
        }
    }
    if (valid && !is_long) finish_column<VEC, L, UPDATE>(A, j, sub, kbase, kact, acc, gw, s2);

    if (A.col_part != nullptr) {
        __shared__ float sh[2 * FM_WAVES];
        const float t0 = fm_wave_sum(wsq);
        const float t1 = fm_wave_sum(vsq);
        if (lane == 0) {
            sh[wave] = t0;
            sh[FM_WAVES + wave] = t1;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            float u0 = 0.f, u1 = 0.f;
#pragma unroll
            for (int wv = 0; wv < FM_WAVES; ++wv) {
                u0 += sh[wv];
                u1 += sh[FM_WAVES + wv];
            }
            A.col_part[2 * (int64_t)blockIdx.x] = u0;
            A.col_part[2 * (int64_t)blockIdx.x + 1] = u1;
        }
    }
}

// One group per segment of a long column: partial sums only.
template <int VEC, int L>
__global__ __launch_bounds__(FM_BLOCK) void k_cols_long(const ColArgs A)
{
    constexpr int R = FM_WAVE / L;
    const int lane = threadIdx.x & (FM_WAVE - 1);
    const int wave = threadIdx.x / FM_WAVE;
    const int sub = lane & (L - 1);
    const int grp = lane / L;
    const int64_t it = A.item_base + (int64_t)blockIdx.x * (FM_WAVES * R) + wave * R + grp;
    const bool valid = it < A.item_base + A.nitems;
    int64_t beg = 0, end = 0;
    if (valid) {
        beg = A.item_beg[it];
        end = beg + A.item_len[it];
    }
    const int kbase = sub * VEC;
    const bool kact = kbase < A.K;
    float acc[VEC];
#pragma unroll
    for (int z = 0; z < VEC; ++z) acc[z] = 0.f;
    float gw = 0.f, s2 = 0.f;
    accumulate_entries<VEC, L>(A, beg, end, sub, kbase, kact, acc, gw, s2);
    gw = fm_group_sum<L>(gw);
    s2 = fm_group_sum<L>(s2);
    if (valid) {
        if (kact) fm_store_vec<VEC>(A.part_acc + it * A.K + kbase, acc);
        if (sub == 0) A.part_gs[it] = make_float2(gw, s2);
    }
}

// One workgroup per long column: group g adds items g, g+NG, g+2NG, ... in fp64,
// the NG group totals are then added in ascending g by group 0, which finishes the column.
template <int VEC, int L, bool UPDATE>
__global__ __launch_bounds__(FM_BLOCK) void k_cols_finish(const ColArgs A)
{
    constexpr int NG = FM_BLOCK / L;  // groups per workgroup
    const int sub = threadIdx.x & (L - 1);
    const int grp = threadIdx.x / L;
    const int64_t lc = A.long_base + blockIdx.x;
    const int64_t j = A.long_col[lc];
    const int64_t first = A.long_first[lc], last = A.long_first[lc + 1];
    const int kbase = sub * VEC;
    const bool kact = kbase < A.K;
    double acc[VEC];
#pragma unroll
    for (int z = 0; z < VEC; ++z) acc[z] = 0.0;
    double gw = 0.0, s2 = 0.0;
    for (int64_t it = first + grp; it < last; it += NG) {
        if (kact) {
            float p[VEC];
            fm_load_vec<VEC>(A.part_acc + it * A.K + kbase, p);
#pragma unroll
            for (int z = 0; z < VEC; ++z) acc[z] += (double)p[z];
        }
        const float2 gs = A.part_gs[it];
        gw += (double)gs.x;
        s2 += (double)gs.y;
    }
    __shared__ double sh[FM_BLOCK * VEC + 2 * NG];
    double* sh_gs = sh + FM_BLOCK * VEC;
#pragma unroll
    for (int z = 0; z < VEC; ++z) sh[(grp * L + sub) * VEC + z] = acc[z];
    if (sub == 0) {
        sh_gs[2 * grp] = gw;
        sh_gs[2 * grp + 1] = s2;
    }
    __syncthreads();
    if (grp == 0) {
        double tot[VEC];
#pragma unroll
        for (int z = 0; z < VEC; ++z) tot[z] = 0.0;
        double tg = 0.0, ts = 0.0;
        for (int g = 0; g < NG; ++g) {
#pragma unroll
            for (int z = 0; z < VEC; ++z) tot[z] += sh[(g * L + sub) * VEC + z];
            tg += sh_gs[2 * g];
            ts += sh_gs[2 * g + 1];
        }
        float accf[VEC];
#pragma unroll
        for (int z = 0; z < VEC; ++z) accf[z] = (float)tot[z];
        finish_column<VEC, L, UPDATE>(A, j, sub, kbase, kact, accf, (float)tg, (float)ts);
    }
}

template <int VEC, int L>
int launch_cols_t(fm_matrix* m, const ColArgs& A, bool update, hipStream_t st)
{
    constexpr int R = FM_WAVE / L;
    const int64_t per = FM_WAVES * R;
    const int64_t grid = (A.D + per - 1) / per;
    if (grid > 0x7fffffffLL || A.nlong > 0x7fffffffLL) return fm_fail(m, FM_ERANGE, "column grid too large");
    if (grid > 0) {
        ProfScope ps(m, st, FMK_COLS);
        if (update)
            hipLaunchKernelGGL((k_cols<VEC, L, true>), dim3((unsigned)grid), dim3(FM_BLOCK), 0, st, A);
        else
            hipLaunchKernelGGL((k_cols<VEC, L, false>), dim3((unsigned)grid), dim3(FM_BLOCK), 0, st, A);
        FM_HIP(m, hipGetLastError());
    }
    if (A.nitems > 0) {
        const int64_t g2 = (A.nitems + per - 1) / per;
        if (g2 > 0x7fffffffLL) return fm_fail(m, FM_ERANGE, "item grid too large");
        {
            ProfScope ps(m, st, FMK_COLS_LONG);
            hipLaunchKernelGGL((k_cols_long<VEC, L>), dim3((unsigned)g2), dim3(FM_BLOCK), 0, st, A);
            FM_HIP(m, hipGetLastError());
        }
        {
            ProfScope ps(m, st, FMK_COLS_FINISH);
            if (update)
                hipLaunchKernelGGL((k_cols_finish<VEC, L, true>), dim3((unsigned)A.nlong), dim3(FM_BLOCK), 0, st, A);
            else
                hipLaunchKernelGGL((k_cols_finish<VEC, L, false>), dim3((unsigned)A.nlong), dim3(FM_BLOCK), 0, st, A);
            FM_HIP(m, hipGetLastError());
        }
    }
    return FM_OK;
}

template <int VEC>
int launch_cols_v(fm_matrix* m, int lanes, const ColArgs& A, bool update, hipStream_t st)
{
    switch (lanes) {
        case 1: return launch_cols_t<VEC, 1>(m, A, update, st);
        case 2: return launch_cols_t<VEC, 2>(m, A, update, st);
        case 4: return launch_cols_t<VEC, 4>(m, A, update, st);
        case 8: return launch_cols_t<VEC, 8>(m, A, update, st);
        case 16: return launch_cols_t<VEC, 16>(m, A, update, st);
        case 32: return launch_cols_t<VEC, 32>(m, A, update, st);
        case 64: return launch_cols_t<VEC, 64>(m, A, update, st);
    }
    return fm_fail(m, FM_EINVAL, "unsupported lane count %d", lanes);
}

}  // namespace

int64_t fm_cols_grid(int64_t D, int32_t K)
{
    int vec, lanes;
    if (!fm_shape_for_K(K, &vec, &lanes)) return 0;
    const int64_t per = (int64_t)FM_WAVES * (FM_WAVE / lanes);
    return (D + per - 1) / per;
}

int fm_launch_cols(fm_matrix* m, const ColArgs& A, bool update, hipStream_t st)
{
    int vec, lanes;
    if (!fm_shape_for_K(A.K, &vec, &lanes)) return fm_fail(m, FM_EINVAL, "unsupported K=%d", A.K);
    switch (vec) {
        case 4: return launch_cols_v<4>(m, lanes, A, update, st);
        case 2: return launch_cols_v<2>(m, lanes, A, update, st);
        default: return launch_cols_v<1>(m, lanes, A, update, st);
    }
}
