// Dense matrices: when every row stores all D columns in order, the CSR values are a dense row-major
// N x D matrix X, and the two sparse products of the pass are dense contractions:
//   G = X V                (eq. compute_a_jk for all rows at once),
//   X^T (r . G)            (the sum over the examples in eq. updates_v),
// which run on the fp32 matrix cores (v_mfma_f32_32x32x2_f32: full fp32 products and sums).  The
// column indices are never read.  Everything else (predictions, loss, multipliers, the fixed-order
// fp64 finish of the partial sums, the fused step) is shared with the sparse path.
//
// Operand layout of the 32x32x2 tile C[32 x 32] += A[32 x 2] B[2 x 32] over the 64 lanes of a wavefront:
//   A: lane l holds A[l % 32][l / 32];   B: lane l holds B[l / 32][l % 32];
//   C: register v of lane l holds C[8 * (v / 4) + 4 * (l / 32) + v % 4][l % 32].
#include "fm_device.h"
#include "fm_internal.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int DT = 32;  // rows (forward) or columns (gradient) per tile
constexpr int FM_DENSE_TILES = 8;      // 32-row tiles per wavefront of the forward kernel
constexpr int FM_DENSE_CHUNKS = 4096;  // row chunks (one wavefront each) of the column kernel

__device__ __forceinline__ int c_row(int v, int lane) { return 8 * (v / 4) + 4 * (lane / 32) + (v % 4); }

// bad[0] = 1 unless rowptr[i] == i * D and col[e] == e % D everywhere
__global__ void k_dense_check(const int64_t* __restrict__ rowptr, const int32_t* __restrict__ col, int64_t N, int64_t D,
                              int32_t* __restrict__ bad)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < N * D && col[e] != (int32_t)(e % D)) bad[0] = 1;
    if (e <= N && rowptr[e] != e * D) bad[0] = 1;
}

// Forward pass over 32 rows per wavefront.  DB = D / 32, KB = K / 32.
// LDS: w (D floats), squared row norms of V (D floats), then one tile of 32 x S floats per wavefront,
// S = max(D, K) + 1 (odd: the column-wise reads of the tile spread over the banks).
template <int DB, int KB>
__global__ __launch_bounds__(FM_BLOCK) void k_rows_dense(const RowArgs A)
{
    constexpr int D = DB * DT, K = KB * DT;
    constexpr int S = (D > K ? D : K) + 1;
    extern __shared__ float lds[];
    float* __restrict__ wl = lds;
    float* __restrict__ nvl = lds + D;
    const int lane = threadIdx.x & (FM_WAVE - 1);
    const int wave = threadIdx.x / FM_WAVE;
    float* __restrict__ tile = lds + 2 * D + wave * (DT * S);
    for (int j = threadIdx.x; j < D; j += FM_BLOCK) {
        wl[j] = A.w[j];
        float n2 = 0.f;
        for (int k = 0; k < K; ++k) {
            const float v = A.V[(int64_t)j * K + k];
            n2 += v * v;
        }
        nvl[j] = n2;
    }
    __syncthreads();
    const int half = lane / 32, lo = lane % 32;
    // B operands: V[2t + half][kb * 32 + lo] for every step t
    float vb[KB][D / 2];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int t = 0; t < D / 2; ++t) vb[kb][t] = A.V[(int64_t)(2 * t + half) * K + kb * DT + lo];

    // A wavefront takes FM_DENSE_TILES consecutive 32-row tiles, so that its share of V is loaded once for all of
    // them.  A tile's rows are contiguous in memory: coalesced float4 loads (rows past the end are zero), issued one
    // tile ahead so that they are in flight while the tile before is worked on.
    constexpr int NC = DT * (D / 4) / FM_WAVE;  // float4 per lane and tile
    const int64_t tile0 = ((int64_t)blockIdx.x * FM_WAVES + wave) * FM_DENSE_TILES;
    float4 xr[NC];
    auto load_tile = [&](int64_t t) {
        const int64_t r0 = t * DT;
        const int64_t left = A.N - r0;
        const int n4 = left <= 0 ? 0 : (int)((left < DT ? left : DT) * (D / 4));
        const float4* __restrict__ src = reinterpret_cast<const float4*>(A.val + (left <= 0 ? 0 : r0 * D));
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            const int c = lane + i * FM_WAVE;
            xr[i] = c < n4 ? src[c] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    load_tile(tile0);
#pragma unroll 1
    for (int tt = 0; tt < FM_DENSE_TILES; ++tt) {
    const int64_t tid = tile0 + tt;
    const int64_t row0 = tid * DT;
    if (row0 >= A.N) return;  // whole wavefronts leave; no barrier follows
    const int nrows = (int)((A.N - row0) < DT ? (A.N - row0) : DT);
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        const int c = lane + i * FM_WAVE;
        const int r = c / (D / 4), k = (c % (D / 4)) * 4;
        float* d = tile + r * S + k;
        d[0] = xr[i].x;
        d[1] = xr[i].y;
        d[2] = xr[i].z;
        d[3] = xr[i].w;
    }
    if (tt + 1 < FM_DENSE_TILES) load_tile(tid + 1);
    __builtin_amdgcn_wave_barrier();
    f32x16 acc[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[kb][v] = 0.f;
    float a_part = 0.f, q_part = 0.f;  // this lane: row lo, columns of parity `half`
#pragma unroll
    for (int t = 0; t < D / 2; ++t) {
        const int k = 2 * t + half;
        const float x = tile[lo * S + k];
        a_part += x * wl[k];
        q_part += (x * x) * nvl[k];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) acc[kb] = __builtin_amdgcn_mfma_f32_32x32x2f32(x, vb[kb][t], acc[kb], 0, 0, 0);
    }
    __builtin_amdgcn_wave_barrier();
    // G tile into LDS (the X tile is no longer needed)
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) tile[c_row(v, lane) * S + kb * DT + lo] = acc[kb][v];
    __builtin_amdgcn_wave_barrier();
    float pair = 0.f;
#pragma unroll
    for (int k = 0; k < K / 2; ++k) {
        const float g = tile[lo * S + half * (K / 2) + k];
        pair += g * g;
    }
    const float a_i = a_part + __shfl_xor(a_part, 32, FM_WAVE);
    const float q_i = q_part + __shfl_xor(q_part, 32, FM_WAVE);
    pair += __shfl_xor(pair, 32, FM_WAVE);
    float l_i = 0.f, r_i = 0.f;
    if (half == 0 && lo < nrows) {
        const int64_t row = row0 + lo;
        const float yh = A.w0[0] + a_i + 0.5f * (pair - q_i);
        if (A.yhat != nullptr) A.yhat[row] = yh;
        if (A.y != nullptr) loss_and_multiplier(A.loss, A.s, yh, A.y[row], l_i, r_i);
        if (A.a != nullptr) A.a[row * A.ss] = a_i;
        if (A.q != nullptr) A.q[row * A.ss] = q_i;
        if (A.y != nullptr && A.r != nullptr) A.r[row * A.ss] = r_i;
    }
    if (A.G != nullptr) {
        for (int c = lane; c < nrows * (K / 4); c += FM_WAVE) {
            const int r = c / (K / 4), k = (c % (K / 4)) * 4;
            const float* s = tile + r * S + k;
            *reinterpret_cast<float4*>(A.G + (row0 + r) * A.gs + k) = make_float4(s[0], s[1], s[2], s[3]);
        }
    }
    if (A.row_part != nullptr) {  // one pair per 32-row tile, lanes added in a fixed order
        const float ls = fm_wave_sum(l_i);
        const float rs = fm_wave_sum(r_i);
        if (lane == 0) {
            A.row_part[2 * tid] = ls;
            A.row_part[2 * tid + 1] = rs;
        }
    }
    __builtin_amdgcn_wave_barrier();  // the next tile overwrites the LDS tile
    }  // tiles of this wavefront
}

// Partial sums of every column over one chunk of rows per wavefront: for column j and latent k
//   acc = sum_i x_ij r_i G_ik,  gw = sum_i x_ij r_i,  s2 = sum_i x_ij^2 r_i      (eqs. updates_w, updates_v),
// two rows per matrix-core step (row parity = the contraction index).  Stored as the row
// [acc | gw | s2] of item j * nchunks + c, which the finish kernels add in fp64 in item order.
template <int DB, int KB>
__global__ __launch_bounds__(FM_BLOCK) void k_cols_dense(const ColArgs A)
{
    constexpr int D = DB * DT, K = KB * DT;
    const int lane = threadIdx.x & (FM_WAVE - 1);
    const int wave = threadIdx.x / FM_WAVE;
    const int half = lane / 32, lo = lane % 32;
    const int64_t c = (int64_t)blockIdx.x * FM_WAVES + wave;
    if (c >= A.nchunks) return;
    const int64_t beg = c * A.chunk_rows;
    const int64_t end = (beg + A.chunk_rows) < A.N ? (beg + A.chunk_rows) : A.N;
    f32x16 acc[DB][KB];
#pragma unroll
    for (int jb = 0; jb < DB; ++jb)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[jb][kb][v] = 0.f;
    float gw[DB], s2[DB];
#pragma unroll
    for (int jb = 0; jb < DB; ++jb) gw[jb] = s2[jb] = 0.f;
    constexpr int U = 4;  // row pairs whose loads are issued together
    for (int64_t r0 = beg; r0 < end; r0 += 2 * U) {
        float x[U][DB], g[U][KB], rr[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t row = r0 + 2 * u + half;
            const bool ok = row < end;
            const int64_t rc = ok ? row : beg;  // a valid row; its contribution is zeroed below
            rr[u] = ok ? A.r[rc * A.rs] : 0.f;
#pragma unroll
            for (int jb = 0; jb < DB; ++jb) x[u][jb] = ok ? A.X[rc * D + jb * DT + lo] : 0.f;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) g[u][kb] = ok ? A.G[rc * A.gs + kb * DT + lo] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) g[u][kb] *= rr[u];
#pragma unroll
            for (int jb = 0; jb < DB; ++jb) {
                const float xr = x[u][jb] * rr[u];
                gw[jb] += xr;
                s2[jb] += x[u][jb] * xr;
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
                    acc[jb][kb] = __builtin_amdgcn_mfma_f32_32x32x2f32(x[u][jb], g[u][kb], acc[jb][kb], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int jb = 0; jb < DB; ++jb) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t j = jb * DT + c_row(v, lane);
            float* __restrict__ row = A.part + (j * A.nchunks + c) * A.ps;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) row[kb * DT + lo] = acc[jb][kb][v];
        }
        const float gt = gw[jb] + __shfl_xor(gw[jb], 32, FM_WAVE);
        const float st = s2[jb] + __shfl_xor(s2[jb], 32, FM_WAVE);
        if (half == 0) {
            float* __restrict__ row = A.part + ((int64_t)(jb * DT + lo) * A.nchunks + c) * A.ps;
            row[K] = gt;
            row[K + 1] = st;
        }
    }
}

template <int DB, int KB>
int launch_rows_dense_t(fm_matrix* m, const RowArgs& A, hipStream_t st)
{
    constexpr int D = DB * DT, K = KB * DT;
    constexpr int S = (D > K ? D : K) + 1;
    const size_t lds = (size_t)(2 * D + FM_WAVES * DT * S) * sizeof(float);
    const int64_t tiles = (A.N + DT - 1) / DT;
    const int64_t per = (int64_t)FM_WAVES * FM_DENSE_TILES;
    const int64_t grid = (tiles + per - 1) / per;
    if (grid > 0x7fffffffLL) return fm_fail(m, FM_ERANGE, "row grid too large");
    ProfScope ps(m, st, FMK_ROWS_FORWARD);
    hipLaunchKernelGGL((k_rows_dense<DB, KB>), dim3((unsigned)grid), dim3(FM_BLOCK), lds, st, A);
    FM_HIP(m, hipGetLastError());
    return FM_OK;
}

template <int DB, int KB>
int launch_cols_dense_t(fm_matrix* m, const ColArgs& A, hipStream_t st)
{
    const int64_t grid = (A.nchunks + FM_WAVES - 1) / FM_WAVES;
    if (grid > 0x7fffffffLL) return fm_fail(m, FM_ERANGE, "chunk grid too large");
    hipLaunchKernelGGL((k_cols_dense<DB, KB>), dim3((unsigned)grid), dim3(FM_BLOCK), 0, st, A);
    FM_HIP(m, hipGetLastError());
    return FM_OK;
}

__global__ void k_dense_index(int64_t D, int64_t nchunks, int32_t* __restrict__ long_col, int64_t* __restrict__ long_first,
                              int32_t* __restrict__ vlong)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j <= D) long_first[j] = j * nchunks;
    if (j < D) {
        long_col[j] = (int32_t)j;
        vlong[j] = (int32_t)j;
    }
}

}  // namespace

int fm_dense_detect(fm_matrix* m, hipStream_t st)
{
    m->is_dense = false;
    const int64_t N = m->N, D = m->D;
    if (N <= 0 || D <= 0 || D > 0x7fffffffLL / 2 || m->nnz != N * D) return FM_OK;
    int32_t* bad = nullptr;
    FM_TRY(fm_dev_alloc(m, (void**)&bad, sizeof(int32_t)));
    int32_t h_bad = 1;
    hipError_t e = hipMemsetAsync(bad, 0, sizeof(int32_t), st);
    if (e == hipSuccess) {
        const int64_t n = m->nnz > N + 1 ? m->nnz : N + 1;
        hipLaunchKernelGGL(k_dense_check, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                           (const int64_t*)m->rowptr, (const int32_t*)m->col, N, D, bad);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpyAsync(&h_bad, bad, sizeof(int32_t), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    fm_dev_free(m, bad);
    if (e != hipSuccess) return fm_fail(m, FM_EHIP, "dense check failed: %s", hipGetErrorString(e));
    m->is_dense = h_bad == 0;
    return FM_OK;
}

// D and K in {32, 64}: the tiles are 32 wide and the accumulators of both kernels stay in registers
bool fm_dense_shape_ok(const fm_matrix* m, int32_t K)
{
    return m->is_dense && m->opt.dense_rows && (m->D == 32 || m->D == 64) && (K == 32 || K == 64);
}

// One chunk of rows per wavefront, FM_DENSE_CHUNKS of them (16 wavefronts per compute unit; with fewer the
// kernel hides less latency than the shorter finish saves); the index says
// that the partial sums of column j are the items j * nchunks .. (j+1) * nchunks - 1.
int fm_dense_build_index(fm_matrix* m, hipStream_t st)
{
    LongIndex* li = &m->ldense;
    if (li->long_col != nullptr || !m->is_dense) return FM_OK;
    const int64_t N = m->N, D = m->D;
    int64_t rows = (N + FM_DENSE_CHUNKS - 1) / FM_DENSE_CHUNKS;
    rows = std::max<int64_t>(64, (rows + 7) / 8 * 8);
    m->dense_chunk_rows = rows;
    m->dense_chunks = (N + rows - 1) / rows;
    FM_TRY(fm_dev_alloc(m, (void**)&li->long_col, (size_t)D * sizeof(int32_t)));
    FM_TRY(fm_dev_alloc(m, (void**)&li->long_first, (size_t)(D + 1) * sizeof(int64_t)));
    FM_TRY(fm_dev_alloc(m, (void**)&li->vlong, (size_t)D * sizeof(int32_t)));
    hipLaunchKernelGGL(k_dense_index, dim3((unsigned)((D + 256) / 256)), dim3(256), 0, st, D, m->dense_chunks, li->long_col,
                       li->long_first, li->vlong);
    FM_HIP(m, hipGetLastError());
    FM_HIP(m, hipStreamSynchronize(st));
    li->nlong = D;
    li->nitems = D * m->dense_chunks;
    li->nvlong = m->dense_chunks > m->tune.vlong ? D : 0;  // a workgroup per column in the finish step
    li->h_long_off.assign({0, li->nlong});
    li->h_item_off.assign({0, li->nitems});
    li->h_short_off.assign({0, 0});
    return FM_OK;
}

int fm_launch_rows_dense(fm_matrix* m, const RowArgs& A, hipStream_t st)
{
    const int db = A.dense_D / DT, kb = A.K / DT;
    if (A.dense_D != db * DT || A.K != kb * DT) return fm_fail(m, FM_EINVAL, "dense kernels need D and K in {32, 64}");
    if (db == 1 && kb == 1) return launch_rows_dense_t<1, 1>(m, A, st);
    if (db == 1 && kb == 2) return launch_rows_dense_t<1, 2>(m, A, st);
    if (db == 2 && kb == 1) return launch_rows_dense_t<2, 1>(m, A, st);
    if (db == 2 && kb == 2) return launch_rows_dense_t<2, 2>(m, A, st);
    return fm_fail(m, FM_EINVAL, "dense kernels need D and K in {32, 64}");
}

int fm_launch_cols_dense(fm_matrix* m, const ColArgs& A, hipStream_t st)
{
    const int db = (int)(A.D / DT), kb = A.K / DT;
    if (A.D != db * DT || A.K != kb * DT || A.X == nullptr || A.nchunks <= 0 || A.chunk_rows <= 0 ||
        A.chunk_rows % 2 != 0)
        return fm_fail(m, FM_EINVAL, "bad arguments of the dense column pass");
    if (db == 1 && kb == 1) return launch_cols_dense_t<1, 1>(m, A, st);
    if (db == 1 && kb == 2) return launch_cols_dense_t<1, 2>(m, A, st);
    if (db == 2 && kb == 1) return launch_cols_dense_t<2, 1>(m, A, st);
    if (db == 2 && kb == 2) return launch_cols_dense_t<2, 2>(m, A, st);
    return fm_fail(m, FM_EINVAL, "dense kernels need D and K in {32, 64}");
}
