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
// Columns longer than `seg` entries are cut into items: k_cols skips them, k_cols_long
// writes one partial sum per item, and the finish kernels add the partials of a column
// in a fixed order, so results are bit-reproducible from run to run.  Items of heavy
// columns are cut at row-panel boundaries and handed out panel by panel, one panel at a
// time per XCD, so that the gathered rows of G stay in that XCD's L2.
#include "fm_device.h"
#include "fm_internal.h"

namespace {

// Accumulate one run of entries [beg,end) of a column into acc/gw/s2 (per-lane
// partials for gw, s2; complete sums for acc's latent slice).
template <int VEC, int L, int PACKED, bool NT, bool LEAN = false>
__device__ __forceinline__ void accumulate_entries(const ColArgs& A, int64_t beg, int64_t end, int sub, int kbase,
                                                   bool kact, float (&acc)[VEC], float& gw, float& s2)
{
    if constexpr (PACKED == FM_PACKED_LANE) {
        // every lane reads inside the row: lanes past the scalars re-read its last VEC floats
        const int last = (int)A.gs - VEC;
        fm_col_accumulate_packed<VEC, L, NT>(A.row, A.val, beg, end, A.G, A.gs, sub, kbase < last ? kbase : last,
                                             A.K / VEC, acc, gw, s2);
    } else {
        const float* __restrict__ r = A.r;
        const int64_t rs = A.rs;
        float unused = 0.f;
        fm_gather_accumulate<VEC, L, false, LEAN ? 1 : FmChunk<L>::CH>(A.row, A.val, beg, end, A.G, A.gs, sub, kact ? kbase : 0, acc, unused,
                                            [&](int i, float x) {
                                                const float xr = x * r[(int64_t)i * rs];
                                                gw += xr;
                                                s2 += x * xr;
                                                return xr;
                                            });
    }
}

// The class of column j that decides which row block it meets in which stratum: its column block in
// the ring of Section 4.2, or the worker it was placed at when columns travel one by one (Section 4.3).
__device__ __forceinline__ int32_t column_class(const ColArgs& A, int64_t j)
{
    if (A.rho == nullptr || A.batch) return 0;
    return A.place != nullptr ? A.place[j] : fm_block_of(j, A.D, A.P);
}

// Share of the regulariser that the step of stratum t applies to a column of class qb.
__device__ __forceinline__ float reg_share(const ColArgs& A, int32_t qb, int32_t t)
{
    if (A.rho == nullptr) return 1.f;
    if (A.batch) return A.rho[t];
    int32_t p = (qb - t) % A.P;
    if (p < 0) p += A.P;
    return A.rho[p];
}

// A column with no entries in its cell only feels the regulariser: x <- x - eta rho lambda x,
// taken as one rounded multiplication by c = 1 - eta (rho lambda).
__device__ __forceinline__ float step_factor(float rho, float lambda, float eta)
{
    return __fsub_rn(1.f, __fmul_rn(eta, __fmul_rn(rho, lambda)));
}

__device__ __forceinline__ double pow_int(double c, uint32_t n)
{
    double r = 1.0;
    while (n != 0) {
        if (n & 1u) r *= c;
        c *= c;
        n >>= 1;
    }
    return r;
}

// Postponed regulariser-only steps t0 .. t1-1 of a column of column block qb, as one factor each
// for v_j and w_j.  The floor split makes row blocks of two sizes only, so the steps have two
// factors only, and the run is  c_small^(n - n_big) * c_big^(n_big)  with n_big read off the block
// bounds; the product is formed in fp64 and rounded once, which is closer to the exact product than
// the n rounded multiplications of steps taken one by one (a single step gives its factor exactly).
__device__ __forceinline__ void catch_up_factors(const ColArgs& A, int32_t qb, int32_t t0, int32_t t1, float& fv,
                                                 float& fw)
{
    fv = fw = 1.f;
    const int32_t n = t1 - t0;
    if (n <= 0) return;
    if (A.rho == nullptr) {  // every step applies the whole regulariser
        fv = (float)pow_int((double)step_factor(1.f, A.lambda_v, A.eta), (uint32_t)n);
        fw = (float)pow_int((double)step_factor(1.f, A.lambda_w, A.eta), (uint32_t)n);
        return;
    }
    int64_t rows;  // rows of the row blocks that the steps t0 .. t1-1 act on
    if (A.batch) {
        rows = A.rb[t1] - A.rb[t0];
    } else {  // blocks p0, p0-1, ..., cyclically
        int32_t p0 = (qb - t0) % A.P;
        if (p0 < 0) p0 += A.P;
        const int32_t lo = p0 - n + 1;
        rows = lo >= 0 ? A.rb[p0 + 1] - A.rb[lo] : (A.rb[p0 + 1] - A.rb[0]) + (A.rb[A.P] - A.rb[A.P + lo]);
    }
    const int64_t base = A.N / A.P;  // rows of a small block; a big one has one more
    const uint32_t n_big = (uint32_t)(rows - (int64_t)n * base);
    const uint32_t n_small = (uint32_t)n - n_big;
    fv = (float)(pow_int((double)step_factor(A.rho_small, A.lambda_v, A.eta), n_small) *
                 pow_int((double)step_factor(A.rho_big, A.lambda_v, A.eta), n_big));
    fw = (float)(pow_int((double)step_factor(A.rho_small, A.lambda_w, A.eta), n_small) *
                 pow_int((double)step_factor(A.rho_big, A.lambda_w, A.eta), n_big));
}

// What the step of column j needs from memory besides the data sums; loaded early by the
// kernels that can, so that it overlaps the gathers.
template <int VEC>
struct ColState {
    float v[VEC];
    float w;
    int32_t t0;  // first stratum whose step the column has not taken yet
};

template <int VEC, bool UPDATE>
__device__ __forceinline__ ColState<VEC> load_column(const ColArgs& A, int64_t j, int sub, int kbase, bool kact)
{
    ColState<VEC> c;
#pragma unroll
    for (int z = 0; z < VEC; ++z) c.v[z] = 0.f;
    c.w = 0.f;
    c.t0 = A.s;
    if (kact) fm_load_vec<VEC>(A.V + j * A.K + kbase, c.v);
    if (sub == 0) c.w = A.w[j];
    if constexpr (UPDATE) {
        if (A.lazy_last != nullptr) c.t0 = A.lazy_last[j];
    }
    return c;
}

// Turn the data sums of column j into the gradient, and either store it or take the
// step (optionally recording the change for the incremental refresh).
template <int VEC, int L, bool UPDATE>
__device__ __forceinline__ void finish_column(const ColArgs& A, int64_t j, int sub, int kbase, bool kact,
                                              const float (&acc)[VEC], float gw, float s2, ColState<VEC> c)
{
    const int K = A.K;
    const int32_t qb = column_class(A, j);
    const float rho = reg_share(A, qb, A.s);
    float fv = 1.f, fw = 1.f;
    if (c.t0 < A.s) catch_up_factors(A, qb, c.t0, A.s, fv, fw);  // postponed regulariser-only steps
    float dn = 0.f;
    if (kact) {
        float g[VEC];
        if (c.t0 < A.s) {
#pragma unroll
            for (int z = 0; z < VEC; ++z) c.v[z] = __fmul_rn(c.v[z], fv);
        }
        const float rl = __fmul_rn(rho, A.lambda_v);
#pragma unroll
        for (int z = 0; z < VEC; ++z) g[z] = __fmaf_rn(rl, c.v[z], __fmaf_rn(-s2, c.v[z], acc[z]));
        if constexpr (UPDATE) {
            float d[VEC], vn[VEC];
#pragma unroll
            for (int z = 0; z < VEC; ++z) {
                d[z] = __fmul_rn(-A.eta, g[z]);
                vn[z] = __fadd_rn(c.v[z], d[z]);
                dn += d[z] * (2.f * c.v[z] + d[z]);  // |v+d|^2 - |v|^2 without cancellation
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
        float wj = c.w;
        if (c.t0 < A.s) wj = __fmul_rn(wj, fw);
        const float g = __fmaf_rn(__fmul_rn(rho, A.lambda_w), wj, gw);
        if constexpr (UPDATE) {
            const float d = __fmul_rn(-A.eta, g);
            A.w[j] = __fadd_rn(wj, d);
            if (A.dwn != nullptr) A.dwn[j] = make_float2(d, dn);
            if (A.lazy_last != nullptr) A.lazy_last[j] = A.s + 1;
            if (A.mark != nullptr) A.mark[j] = 1;  // this column has taken its step from data
        } else {
            if (A.grad_w != nullptr) A.grad_w[j] = g;
        }
    }
}

// Short non-empty columns (1..seg entries), taken from a list: one group per column.
template <int VEC, int L, bool UPDATE, int PACKED>
__global__ __launch_bounds__(FM_BLOCK) void k_cols(const ColArgs A)
{
    constexpr int R = FM_WAVE / L;
    const int lane = threadIdx.x & (FM_WAVE - 1);
    const int wave = threadIdx.x / FM_WAVE;
    const int sub = lane & (L - 1);
    const int grp = lane / L;
    const int64_t pos = (int64_t)blockIdx.x * (FM_WAVES * R) + wave * R + grp;
    const bool valid = pos < A.nshort;
    int64_t j = 0, beg = 0, end = 0;
    if (valid) {
        j = A.short_col[pos];
        if (A.ptr != nullptr) {
            beg = A.ptr[j];
            end = A.ptr[j + 1];
        } else {
            beg = A.short_beg[pos];
            end = beg + A.short_len[pos];
        }
    }
    const int kbase = sub * VEC;
    const bool kact = kbase < A.K;
    // the column's own values do not depend on the gathers: fetch them first
    const ColState<VEC> c = load_column<VEC, UPDATE>(A, j, sub, kbase, kact && valid);
    float acc[VEC];
#pragma unroll
    for (int z = 0; z < VEC; ++z) acc[z] = 0.f;
    float gw = 0.f, s2 = 0.f;
    // short columns: no reuse of the gathered rows.  Wide groups (few columns per wavefront) take
    // the lean loop: fewer registers, so more wavefronts and more columns in flight.
    accumulate_entries<VEC, L, PACKED, true, (L >= 16)>(A, beg, end, sub, kbase, kact, acc, gw, s2);
    gw = fm_group_sum<L>(gw);
    s2 = fm_group_sum<L>(s2);
    if (valid) finish_column<VEC, L, UPDATE>(A, j, sub, kbase, kact, acc, gw, s2, c);
}

// Columns with nothing stored (in this matrix or stratum) only feel the regulariser; one group
// of LE = K/VEC lanes per column over all D columns, consecutive groups on consecutive columns
// so that V is streamed.  The gradient is finish_column with zero data sums; the step is the
// multiplication by the step factor.  A group takes FM_EMPTY_U columns, one from each of as many
// consecutive slabs of columns: the tests for emptiness are all issued before the first row of V
// is asked for, and all rows before the first is written, so that the kernel is not one memory
// round trip after the other per column.
constexpr int FM_EMPTY_U = 4;
template <int VEC, int LE, bool UPDATE>
__global__ __launch_bounds__(FM_BLOCK) void k_cols_empty(const ColArgs A)
{
    constexpr int R = FM_WAVE / LE;
    constexpr int U = FM_EMPTY_U;
    const int lane = threadIdx.x & (FM_WAVE - 1);
    const int wave = threadIdx.x / FM_WAVE;
    const int sub = lane & (LE - 1);
    const int grp = lane / LE;
    const int kbase = sub * VEC;
    const bool kact = kbase < A.K;
    int64_t j[U];
    bool todo[U];  // uniform inside a group
#pragma unroll
    for (int u = 0; u < U; ++u) {
        j[u] = ((int64_t)blockIdx.x * U + u) * (FM_WAVES * R) + wave * R + grp;
        todo[u] = j[u] < A.D;
        if (todo[u]) {
            if (A.ptr != nullptr) {
                todo[u] = A.ptr[j[u] + 1] == A.ptr[j[u]];
            } else {  // a stratum or batch: the columns with entries marked themselves; the marks are left clear
                const bool marked = A.mark[j[u]] != 0;
                if (marked && sub == 0) A.mark[j[u]] = 0;
                todo[u] = !marked;
            }
        }
    }
    if constexpr (!UPDATE) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (!todo[u]) continue;
            float acc[VEC];
#pragma unroll
            for (int z = 0; z < VEC; ++z) acc[z] = 0.f;
            finish_column<VEC, LE, false>(A, j[u], sub, kbase, kact, acc, 0.f, 0.f,
                                          load_column<VEC, false>(A, j[u], sub, kbase, kact));
        }
    } else {
        float v[U][VEC];
        float wj[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int z = 0; z < VEC; ++z) v[u][z] = 0.f;
            wj[u] = 0.f;
            if (todo[u] && kact) fm_load_vec<VEC>(A.V + j[u] * A.K + kbase, v[u]);
            if (todo[u] && sub == 0) wj[u] = A.w[j[u]];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (!todo[u]) continue;
            const int32_t qb = column_class(A, j[u]);
            const float rho = reg_share(A, qb, A.s);
            float dn = 0.f;
            if (kact) {
                const float f = step_factor(rho, A.lambda_v, A.eta);
                float vn[VEC], d[VEC];
#pragma unroll
                for (int z = 0; z < VEC; ++z) {
                    vn[z] = __fmul_rn(v[u][z], f);
                    d[z] = vn[z] - v[u][z];
                    dn += d[z] * (2.f * v[u][z] + d[z]);
                }
                fm_store_vec<VEC>(A.V + j[u] * A.K + kbase, vn);
                if (A.dV != nullptr) fm_store_vec<VEC>(A.dV + j[u] * A.K + kbase, d);
            }
            if (A.dwn != nullptr) dn = fm_group_sum<LE>(dn);
            if (sub == 0) {
                const float wn = __fmul_rn(wj[u], step_factor(rho, A.lambda_w, A.eta));
                A.w[j[u]] = wn;
                if (A.dwn != nullptr) A.dwn[j[u]] = make_float2(wn - wj[u], dn);
            }
        }
    }
}

// The postponed regulariser steps of every column, strata lazy_last[j] .. A.s-1; one group of LE
// lanes per column, consecutive columns in consecutive groups.
template <int VEC, int LE>
__global__ __launch_bounds__(FM_BLOCK) void k_cols_flush(const ColArgs A)
{
    constexpr int R = FM_WAVE / LE;
    const int lane = threadIdx.x & (FM_WAVE - 1);
    const int wave = threadIdx.x / FM_WAVE;
    const int sub = lane & (LE - 1);
    const int grp = lane / LE;
    const int64_t j = (int64_t)blockIdx.x * (FM_WAVES * R) + wave * R + grp;
    if (j >= A.D) return;  // whole groups leave together
    const int32_t t0 = A.lazy_last[j];
    if (t0 >= A.s) return;
    const int32_t qb = column_class(A, j);
    float fv, fw;
    catch_up_factors(A, qb, t0, A.s, fv, fw);
    const int kbase = sub * VEC;
    if (kbase < A.K) {
        float v[VEC];
        fm_load_vec<VEC>(A.V + j * A.K + kbase, v);
#pragma unroll
        for (int z = 0; z < VEC; ++z) v[z] = __fmul_rn(v[z], fv);
        fm_store_vec<VEC>(A.V + j * A.K + kbase, v);
    }
    if (sub == 0) A.w[j] = __fmul_rn(A.w[j], fw);
}

// Partial sums of item `it`: one row [acc_0..acc_{K-1} | gw | s2 | pad] of A.ps floats, a whole
// number of 128-byte lines.  Items are written in processing order and read in column order, so
// the rows are scattered: with float4 lanes the group writes the whole row, padding included, so
// that no line is left partly written.
template <int VEC, int L>
__device__ __forceinline__ void store_partial(const ColArgs& A, int64_t it, int sub, int kbase, bool kact,
                                              const float (&acc)[VEC], float gw, float s2)
{
    float* __restrict__ row = A.part + it * A.ps;
    if constexpr (VEC == 4) {
        for (int o = sub * 4; o < A.ps; o += L * 4) {
            float z[4] = {0.f, 0.f, 0.f, 0.f};
            if (o < A.K) {
#pragma unroll
                for (int t = 0; t < 4; ++t) z[t] = acc[t];  // first pass only: o == kbase
            } else if (o == A.K) {
                z[0] = gw;
                z[1] = s2;
            }
            fm_store_vec<4>(row + o, z);
        }
    } else {
        if (kact) fm_store_vec<VEC>(row + kbase, acc);
        if (sub == 0) {
            row[A.K] = gw;
            row[A.K + 1] = s2;
        }
    }
}

// One group per item of a long column: partial sums only.  With an order array,
// workgroup b takes its items from list b % FM_XCDS (the XCD it runs on).
template <int VEC, int L, int PACKED>
__global__ __launch_bounds__(FM_BLOCK) void k_cols_long(const ColArgs A)
{
    constexpr int R = FM_WAVE / L;
    const int lane = threadIdx.x & (FM_WAVE - 1);
    const int wave = threadIdx.x / FM_WAVE;
    const int sub = lane & (L - 1);
    const int grp = lane / L;
    const int slot_in_block = wave * R + grp;
    int64_t it = -1;
    int64_t beg = 0, end = 0;
    bool reused = false;  // item of a heavy column inside a panel: its rows are gathered again soon
    if (A.order != nullptr && A.lin_mode) {
        const int64_t rel = (int64_t)blockIdx.x * (FM_WAVES * R) + slot_in_block;
        if (rel < A.lin_count) {
            const int64_t pos = A.lin_base + rel;
            it = A.order[pos];
            beg = A.ord_beg[pos];
            end = beg + A.ord_len[pos];
        }
        reused = true;
    } else if (A.order != nullptr) {
        const int x = blockIdx.x % FM_XCDS;
        const int64_t pos = A.list_off[x] + (int64_t)(blockIdx.x / FM_XCDS) * (FM_WAVES * R) + slot_in_block;
        if (pos < A.list_off[x + 1]) {
            it = A.order[pos];
            beg = A.ord_beg[pos];
            end = beg + A.ord_len[pos];
        }
        reused = pos < A.list_mid[x];
    } else {
        const int64_t pos = (int64_t)blockIdx.x * (FM_WAVES * R) + slot_in_block;
        if (pos < A.nitems) {
            it = A.item_base + pos;
            beg = A.item_beg[it];
            end = beg + A.item_len[it];
        }
    }
    const bool valid = it >= 0;
    const int kbase = sub * VEC;
    const bool kact = kbase < A.K;
    float acc[VEC];
#pragma unroll
    for (int z = 0; z < VEC; ++z) acc[z] = 0.f;
    float gw = 0.f, s2 = 0.f;
    if (reused)
        accumulate_entries<VEC, L, PACKED, false>(A, beg, end, sub, kbase, kact, acc, gw, s2);
    else
        accumulate_entries<VEC, L, PACKED, true>(A, beg, end, sub, kbase, kact, acc, gw, s2);
    gw = fm_group_sum<L>(gw);
    s2 = fm_group_sum<L>(s2);
    if (valid) store_partial<VEC, L>(A, it, sub, kbase, kact, acc, gw, s2);
}

// Dense-ish columns, LDS-staged: workgroup t copies G and r of the tile_rows rows of row tile t
// (packed or planar aggregates) into LDS once, then its groups walk the tile's items
// (pieces of dense-ish columns whose rows lie inside the tile) and gather G and r from LDS.
// One partial sum per item, as in k_cols_long.  L lanes of VEC=4 latent dimensions per group.
template <int L>
__global__ __launch_bounds__(FM_BLOCK) void k_cols_tile(const ColArgs A)
{
    constexpr int VEC = 4;
    constexpr int NG = FM_BLOCK / L;
    extern __shared__ float tile[];  // G part: tile_rows x K floats, then r: tile_rows floats
    const int K = A.K;
    const int S = K;
    float* __restrict__ tile_r = tile + A.tile_rows * K;
    const int chunks = K / VEC;  // float4 chunks of G per row
    const int64_t t = blockIdx.x;
    const int64_t row0 = t * A.tile_rows;
    const int64_t nrows = (A.N - row0) < A.tile_rows ? (A.N - row0) : A.tile_rows;
    {   // copy in batches of eight float4 per thread: all loads of a batch are issued before the first store
        const int total = (int)nrows * chunks;
        const float* __restrict__ src = A.G + row0 * A.gs;
        const float* __restrict__ rsrc = A.r + row0 * A.rs;
        constexpr int U = 8;
        for (int c0 = threadIdx.x; c0 < total; c0 += U * FM_BLOCK) {
            float4 v[U];
            int dst[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = c0 + u * FM_BLOCK;
                const int cc = c < total ? c : total - 1;
                const int rr = cc / chunks, ch = cc - rr * chunks;
                dst[u] = c < total ? (rr << 8) | ch : -1;  // chunks <= 64 for every K of this path
                v[u] = *reinterpret_cast<const float4*>(src + (int64_t)rr * A.gs + ch * VEC);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (dst[u] < 0) continue;
                const int rr = dst[u] >> 8, ch = dst[u] & 255;
                *reinterpret_cast<float4*>(tile + rr * S + ch * VEC) = v[u];
            }
        }
        // r of the rows (a loop of its own: no branch between the loads of a batch above)
        for (int rr = threadIdx.x; rr < (int)nrows; rr += FM_BLOCK) tile_r[rr] = rsrc[(int64_t)rr * A.rs];
    }
    __syncthreads();

    const int sub = threadIdx.x & (L - 1);
    const int grp = threadIdx.x / L;
    const int kbase = sub * VEC;
    const bool kact = kbase < K;
    const int kb = kact ? kbase : 0;
    const int64_t pend = A.tile_ptr[t + 1];
    for (int64_t pos = A.tile_ptr[t] + grp; pos < pend; pos += NG) {
        const int64_t it = A.order[pos];
        const int64_t beg = A.ord_beg[pos];
        const int64_t end = beg + A.ord_len[pos];
        float acc[VEC] = {0.f, 0.f, 0.f, 0.f};
        float gw = 0.f, s2 = 0.f;
        constexpr int CH = FmChunk<L>::CH;
        for (int64_t e = beg; e < end; e += L * CH) {
            int il[CH];
            float xr[CH];
#pragma unroll
            for (int u = 0; u < CH; ++u) {  // own entries: index and value from global memory
                const int64_t my = e + u * L + sub;
                const bool has = my < end;
                const int64_t mc = has ? my : end - 1;
                il[u] = (int)((int64_t)A.row[mc] - row0);
                xr[u] = has ? A.val[mc] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < CH; ++u) {  // r of the own entry from LDS
                const float x = xr[u];
                xr[u] = x * tile_r[il[u]];
                gw += xr[u];
                s2 += x * xr[u];
            }
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                fm_static_for<0, L>([&](auto tc) {
                    constexpr int T = decltype(tc)::value;
                    const int ir = fm_bcast_i<L, T>(il[u]);
                    const float mt = fm_bcast_f<L, T>(xr[u]);
                    const float4 g = *reinterpret_cast<const float4*>(tile + ir * S + kb);
                    acc[0] += mt * g.x;
                    acc[1] += mt * g.y;
                    acc[2] += mt * g.z;
                    acc[3] += mt * g.w;
                });
            }
        }
        gw = fm_group_sum<L>(gw);
        s2 = fm_group_sum<L>(s2);
        store_partial<4, L>(A, it, sub, kbase, kact, acc, gw, s2);
    }
}

// Sum of the partials first, first+step, ... < last of one column, in fp64 and in that
// order; eight loads are issued before the first add so that the loop is not one memory
// round trip per item.
template <int VEC>
__device__ __forceinline__ void add_partials(const ColArgs& A, int64_t first, int64_t last, int64_t step, int kbase,
                                             bool kact, double (&acc)[VEC], double& gw, double& s2)
{
    constexpr int U = 8;
    const int kb = kact ? kbase : 0;
    int64_t it = first;
    for (; it + (U - 1) * step < last; it += U * step) {
        float p[U][VEC];
        float g0[U], g1[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float* __restrict__ row = A.part + (it + u * step) * A.ps;
            fm_load_vec<VEC>(row + kb, p[u]);
            g0[u] = row[A.K];
            g1[u] = row[A.K + 1];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int z = 0; z < VEC; ++z) acc[z] += (double)p[u][z];
            gw += (double)g0[u];
            s2 += (double)g1[u];
        }
    }
    for (; it < last; it += step) {
        const float* __restrict__ row = A.part + it * A.ps;
        float p[VEC];
        fm_load_vec<VEC>(row + kb, p);
#pragma unroll
        for (int z = 0; z < VEC; ++z) acc[z] += (double)p[z];
        gw += (double)row[A.K];
        s2 += (double)row[A.K + 1];
    }
}

// One wavefront per long column: group g adds items g, g+R, g+2R, ...; the R group
// totals are then combined by a fixed butterfly and group 0 finishes the column.
// Columns with more than vlong_items items are left to k_cols_finish_block (if a list
// of them was given).
template <int VEC, int L, bool UPDATE>
__global__ __launch_bounds__(FM_BLOCK) void k_cols_finish_wave(const ColArgs A)
{
    constexpr int R = FM_WAVE / L;
    const int lane = threadIdx.x & (FM_WAVE - 1);
    const int wave = threadIdx.x / FM_WAVE;
    const int sub = lane & (L - 1);
    const int grp = lane / L;
    const int64_t rel = (int64_t)blockIdx.x * FM_WAVES + wave;
    if (rel >= A.nlong) return;  // whole wavefront leaves together
    const int64_t lc = A.long_base + rel;
    const int64_t first = A.long_first[lc], last = A.long_first[lc + 1];
    if (A.vlong != nullptr && last - first > A.vlong_items) return;
    const int64_t j = A.long_col[lc];
    const int kbase = sub * VEC;
    const bool kact = kbase < A.K;
    double acc[VEC];
#pragma unroll
    for (int z = 0; z < VEC; ++z) acc[z] = 0.0;
    double gw = 0.0, s2 = 0.0;
    add_partials<VEC>(A, first + grp, last, R, kbase, kact, acc, gw, s2);
    // combine the R groups: lanes with equal `sub` hold the same latent slice
#pragma unroll
    for (int o = L; o < FM_WAVE; o <<= 1) {
#pragma unroll
        for (int z = 0; z < VEC; ++z) acc[z] += __shfl_xor(acc[z], o, FM_WAVE);
        gw += __shfl_xor(gw, o, FM_WAVE);
        s2 += __shfl_xor(s2, o, FM_WAVE);
    }
    if (grp == 0) {
        float accf[VEC];
#pragma unroll
        for (int z = 0; z < VEC; ++z) accf[z] = (float)acc[z];
        finish_column<VEC, L, UPDATE>(A, j, sub, kbase, kact, accf, (float)gw, (float)s2,
                                      load_column<VEC, UPDATE>(A, j, sub, kbase, kact));
    }
}

// One workgroup per very long column: group g adds items g, g+NG, g+2NG, ... in fp64,
// the NG group totals are then added in ascending g by group 0, which finishes the column.
template <int VEC, int L, bool UPDATE>
__global__ __launch_bounds__(FM_BLOCK) void k_cols_finish_block(const ColArgs A)
{
    constexpr int NG = FM_BLOCK / L;  // groups per workgroup
    const int sub = threadIdx.x & (L - 1);
    const int grp = threadIdx.x / L;
    const int64_t lc = A.vlong[blockIdx.x];
    const int64_t j = A.long_col[lc];
    const int64_t first = A.long_first[lc], last = A.long_first[lc + 1];
    const int kbase = sub * VEC;
    const bool kact = kbase < A.K;
    double acc[VEC];
#pragma unroll
    for (int z = 0; z < VEC; ++z) acc[z] = 0.0;
    double gw = 0.0, s2 = 0.0;
    add_partials<VEC>(A, first + grp, last, NG, kbase, kact, acc, gw, s2);
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
        finish_column<VEC, L, UPDATE>(A, j, sub, kbase, kact, accf, (float)tg, (float)ts,
                                      load_column<VEC, UPDATE>(A, j, sub, kbase, kact));
    }
}

// LDS-staged kernel for the tile items; false if the tile does not fit in LDS for this K
// (the caller then runs the items through k_cols_long).
template <int L>
bool launch_tile_l(fm_matrix* m, const ColArgs& A, size_t lds, hipStream_t st)
{
    constexpr unsigned bit = 1u << __builtin_ctz((unsigned)L);
    if (!(m->tile_attr_set & bit)) {  // opt in once per handle to more than the default 64 KB of dynamic LDS
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_cols_tile<L>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 256) != hipSuccess) {
            (void)hipGetLastError();
            if (lds > 64 * 1024) return false;
        }
        m->tile_attr_set |= bit;
    }
    hipLaunchKernelGGL((k_cols_tile<L>), dim3((unsigned)A.ntiles), dim3(FM_BLOCK), lds, st, A);
    return true;
}

inline bool launch_tile(fm_matrix* m, const ColArgs& A, hipStream_t st)
{
    if (A.ntiles <= 0 || A.ntiles > 0x7fffffffLL || A.K % 4 != 0) return false;
    const size_t lds = (size_t)A.tile_rows * (size_t)(A.K + 1) * sizeof(float);
    // at least two workgroups per compute unit, or the copy of one tile cannot overlap the work on another
    if (lds > 72 * 1024) return false;
    int need = A.K / 4, l = 1;
    while (l < need) l <<= 1;
    switch (l) {
        case 1: return launch_tile_l<1>(m, A, lds, st);
        case 2: return launch_tile_l<2>(m, A, lds, st);
        case 4: return launch_tile_l<4>(m, A, lds, st);
        case 8: return launch_tile_l<8>(m, A, lds, st);
        case 16: return launch_tile_l<16>(m, A, lds, st);
        case 32: return launch_tile_l<32>(m, A, lds, st);
        case 64: return launch_tile_l<64>(m, A, lds, st);
    }
    return false;
}

// k_cols_empty with LE = smallest power of two >= K/VEC lanes per column
template <int VEC, int LE>
int launch_empty_l(fm_matrix* m, const ColArgs& A, bool update, hipStream_t st)
{
    const int64_t per = (int64_t)FM_WAVES * (FM_WAVE / LE) * FM_EMPTY_U;
    const int64_t grid = (A.D + per - 1) / per;
    if (grid > 0x7fffffffLL) return fm_fail(m, FM_ERANGE, "column grid too large");
    if (update)
        hipLaunchKernelGGL((k_cols_empty<VEC, LE, true>), dim3((unsigned)grid), dim3(FM_BLOCK), 0, st, A);
    else
        hipLaunchKernelGGL((k_cols_empty<VEC, LE, false>), dim3((unsigned)grid), dim3(FM_BLOCK), 0, st, A);
    FM_HIP(m, hipGetLastError());
    return FM_OK;
}

template <int VEC>
int launch_empty(fm_matrix* m, const ColArgs& A, bool update, hipStream_t st)
{
    int need = A.K / VEC, l = 1;
    while (l < need) l <<= 1;
    switch (l) {
        case 1: return launch_empty_l<VEC, 1>(m, A, update, st);
        case 2: return launch_empty_l<VEC, 2>(m, A, update, st);
        case 4: return launch_empty_l<VEC, 4>(m, A, update, st);
        case 8: return launch_empty_l<VEC, 8>(m, A, update, st);
        case 16: return launch_empty_l<VEC, 16>(m, A, update, st);
        case 32: return launch_empty_l<VEC, 32>(m, A, update, st);
        case 64: return launch_empty_l<VEC, 64>(m, A, update, st);
    }
    return fm_fail(m, FM_EINVAL, "unsupported K=%d", A.K);
}

template <int VEC, int LE>
int launch_flush_l(fm_matrix* m, const ColArgs& A, hipStream_t st)
{
    const int64_t per = (int64_t)FM_WAVES * (FM_WAVE / LE);
    const int64_t grid = (A.D + per - 1) / per;
    if (grid > 0x7fffffffLL) return fm_fail(m, FM_ERANGE, "column grid too large");
    ProfScope ps(m, st, FMK_COLS);
    hipLaunchKernelGGL((k_cols_flush<VEC, LE>), dim3((unsigned)grid), dim3(FM_BLOCK), 0, st, A);
    FM_HIP(m, hipGetLastError());
    return FM_OK;
}

template <int VEC>
int launch_flush(fm_matrix* m, const ColArgs& A, hipStream_t st)
{
    int need = A.K / VEC, l = 1;
    while (l < need) l <<= 1;
    switch (l) {
        case 1: return launch_flush_l<VEC, 1>(m, A, st);
        case 2: return launch_flush_l<VEC, 2>(m, A, st);
        case 4: return launch_flush_l<VEC, 4>(m, A, st);
        case 8: return launch_flush_l<VEC, 8>(m, A, st);
        case 16: return launch_flush_l<VEC, 16>(m, A, st);
        case 32: return launch_flush_l<VEC, 32>(m, A, st);
        case 64: return launch_flush_l<VEC, 64>(m, A, st);
    }
    return fm_fail(m, FM_EINVAL, "unsupported K=%d", A.K);
}

template <int VEC, int L, int PACKED>
int launch_cols_t(fm_matrix* m, const ColArgs& A, bool update, hipStream_t st)
{
    constexpr int R = FM_WAVE / L;
    const int64_t per = FM_WAVES * R;
    if (A.nlong > 0x7fffffffLL) return fm_fail(m, FM_ERANGE, "column grid too large");
    // The three accumulation kernels touch disjoint columns.  When there are LDS-staged items,
    // k_cols and k_cols_tile go to two side streams so that the LDS-bound kernel overlaps the
    // memory-bound ones; the finish kernels wait for all three.
    const int64_t ntile_items = A.order != nullptr ? A.nitems - A.list_off[FM_XCDS] : 0;
    // columns without entries only feel the regulariser (skipped when there is none and nothing records the
    // change, or when such steps are postponed)
    const bool need_empty =
        (A.lambda_w != 0.f || A.lambda_v != 0.f || !update || A.dV != nullptr) && A.lazy_last == nullptr;
    ColArgs Am = A;
    if (!need_empty || A.ptr != nullptr) Am.mark = nullptr;  // marks are only set when a kernel will clear them
    // (not while per-kernel timing is on: each kernel is then timed alone on the launch stream)
    const bool dense = A.X != nullptr;  // one kernel leaves the partial sums of every column
    const bool side = !dense && (ntile_items > 0 || (A.nitems > 0 && A.nshort > 0)) && !m->prof && fm_side_streams(m);
    hipStream_t s_cols = st, s_tile = st;
    if (side) {
        FM_HIP(m, hipEventRecord(m->ev_fork, st));
        FM_HIP(m, hipStreamWaitEvent(m->side1, m->ev_fork, 0));
        FM_HIP(m, hipStreamWaitEvent(m->side2, m->ev_fork, 0));
        s_tile = m->side1;
        s_cols = m->side2;
    }
    if (dense) {
        ProfScope ps(m, st, FMK_COLS_LONG);
        FM_TRY(fm_launch_cols_dense(m, A, st));
    }
    if (!dense && ntile_items > 0) {  // items of dense-ish columns, sorted by row tile
        ProfScope ps(m, s_tile, FMK_COLS_TILE);
        bool staged = false;
        if constexpr (VEC == 4) staged = launch_tile(m, A, s_tile);
        if (!staged) {  // same items through global memory
            ColArgs B = A;
            B.lin_mode = 1;
            B.lin_base = A.list_off[FM_XCDS];
            B.lin_count = ntile_items;
            const int64_t g4 = (ntile_items + per - 1) / per;
            if (g4 > 0x7fffffffLL) return fm_fail(m, FM_ERANGE, "item grid too large");
            hipLaunchKernelGGL((k_cols_long<VEC, L, PACKED>), dim3((unsigned)g4), dim3(FM_BLOCK), 0, s_tile, B);
        }
        FM_HIP(m, hipGetLastError());
    }
    if (!dense && A.nitems > 0) {
        int64_t g2;
        if (A.order != nullptr) {
            int64_t longest = 0;
            for (int x = 0; x < FM_XCDS; ++x)
                longest = std::max<int64_t>(longest, A.list_off[x + 1] - A.list_off[x]);
            g2 = FM_XCDS * ((longest + per - 1) / per);
        } else {
            g2 = (A.nitems + per - 1) / per;
        }
        if (g2 > 0x7fffffffLL) return fm_fail(m, FM_ERANGE, "item grid too large");
        if (g2 > 0) {
            ProfScope ps(m, st, FMK_COLS_LONG);
            hipLaunchKernelGGL((k_cols_long<VEC, L, PACKED>), dim3((unsigned)g2), dim3(FM_BLOCK), 0, st, A);
            FM_HIP(m, hipGetLastError());
        }
    }
    if (!dense) {
        ProfScope ps(m, s_cols, FMK_COLS);
        const int64_t g1 = (A.nshort + per - 1) / per;
        if (g1 > 0x7fffffffLL) return fm_fail(m, FM_ERANGE, "column grid too large");
        if (g1 > 0) {
            if (update)
                hipLaunchKernelGGL((k_cols<VEC, L, true, PACKED>), dim3((unsigned)g1), dim3(FM_BLOCK), 0, s_cols, Am);
            else
                hipLaunchKernelGGL((k_cols<VEC, L, false, PACKED>), dim3((unsigned)g1), dim3(FM_BLOCK), 0, s_cols, Am);
            FM_HIP(m, hipGetLastError());
        }
        // empty columns of the full matrix: regulariser only (a stratum's wait for the marks, below)
        // (nothing to launch when every column of the matrix is listed as short or long)
        if (need_empty && A.ptr != nullptr && A.D > 0 && A.nshort + A.nlong < A.D)
            FM_TRY((launch_empty<VEC>(m, A, update, s_cols)));
    }
    if (side) {
        FM_HIP(m, hipEventRecord(m->ev_join1, m->side1));
        FM_HIP(m, hipEventRecord(m->ev_join2, m->side2));
        FM_HIP(m, hipStreamWaitEvent(st, m->ev_join1, 0));
        FM_HIP(m, hipStreamWaitEvent(st, m->ev_join2, 0));
    }
    if (A.nitems > 0) {
        {
            ProfScope ps(m, st, FMK_COLS_FINISH);
            const int64_t g3 = (A.nlong + FM_WAVES - 1) / FM_WAVES;
            const bool all_by_block = A.vlong != nullptr && A.nvlong == A.nlong;  // nothing left for the wavefronts
            if (!all_by_block) {
                if (update)
                    hipLaunchKernelGGL((k_cols_finish_wave<VEC, L, true>), dim3((unsigned)g3), dim3(FM_BLOCK), 0, st, Am);
                else
                    hipLaunchKernelGGL((k_cols_finish_wave<VEC, L, false>), dim3((unsigned)g3), dim3(FM_BLOCK), 0, st, Am);
                FM_HIP(m, hipGetLastError());
            }
            if (A.vlong != nullptr && A.nvlong > 0) {
                if (update)
                    hipLaunchKernelGGL((k_cols_finish_block<VEC, L, true>), dim3((unsigned)A.nvlong), dim3(FM_BLOCK),
                                       0, st, Am);
                else
                    hipLaunchKernelGGL((k_cols_finish_block<VEC, L, false>), dim3((unsigned)A.nvlong), dim3(FM_BLOCK),
                                       0, st, Am);
                FM_HIP(m, hipGetLastError());
            }
        }
    }
    // a stratum or batch whose steps are taken at once: every column that had entries has marked itself by now
    if (need_empty && A.ptr == nullptr && A.D > 0) {
        ProfScope ps(m, st, FMK_COLS);
        FM_TRY((launch_empty<VEC>(m, Am, update, st)));
    }
    return FM_OK;
}

template <int VEC, int PACKED>
int launch_cols_v(fm_matrix* m, int lanes, const ColArgs& A, bool update, hipStream_t st)
{
    switch (lanes) {
        case 1: return launch_cols_t<VEC, 1, PACKED>(m, A, update, st);
        case 2: return launch_cols_t<VEC, 2, PACKED>(m, A, update, st);
        case 4: return launch_cols_t<VEC, 4, PACKED>(m, A, update, st);
        case 8: return launch_cols_t<VEC, 8, PACKED>(m, A, update, st);
        case 16: return launch_cols_t<VEC, 16, PACKED>(m, A, update, st);
        case 32: return launch_cols_t<VEC, 32, PACKED>(m, A, update, st);
        case 64: return launch_cols_t<VEC, 64, PACKED>(m, A, update, st);
    }
    return fm_fail(m, FM_EINVAL, "unsupported lane count %d", lanes);
}

}  // namespace

// lanes per column group: K/VEC latent lanes, plus one lane for the scalars of a packed row
// when the row [G | r] lies inside one 128-byte line
static bool cols_shape(int32_t K, int packed, int* vec, int* lanes)
{
    if (!fm_shape_for_K(K, vec, lanes)) return false;
    if (packed == FM_PACKED_LANE) {
        int need = K / 4 + 1, l = 1;
        while (l < need) l <<= 1;
        *lanes = l;
    }
    return true;
}

int fm_launch_cols(fm_matrix* m, const ColArgs& A, bool update, hipStream_t st)
{
    int vec, lanes;
    if (!cols_shape(A.K, A.packed, &vec, &lanes)) return fm_fail(m, FM_EINVAL, "unsupported K=%d", A.K);
    if (A.packed == FM_PACKED_LANE) return launch_cols_v<4, FM_PACKED_LANE>(m, lanes, A, update, st);
    switch (vec) {
        case 4: return launch_cols_v<4, FM_PLANAR>(m, lanes, A, update, st);
        case 2: return launch_cols_v<2, FM_PLANAR>(m, lanes, A, update, st);
        default: return launch_cols_v<1, FM_PLANAR>(m, lanes, A, update, st);
    }
}

int fm_launch_cols_flush(fm_matrix* m, const ColArgs& A, hipStream_t st)
{
    int vec, lanes;
    if (!fm_shape_for_K(A.K, &vec, &lanes)) return fm_fail(m, FM_EINVAL, "unsupported K=%d", A.K);
    if (A.lazy_last == nullptr || A.D <= 0) return FM_OK;
    switch (vec) {
        case 4: return launch_flush<4>(m, A, st);
        case 2: return launch_flush<2>(m, A, st);
        default: return launch_flush<1>(m, A, st);
    }
}
