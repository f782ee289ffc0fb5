// C-ABI entry points and the epoch drivers.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>

#include "fm_internal.h"

static thread_local std::string g_build_error;

int fm_fail(fm_matrix* m, int code, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    if (m != nullptr) m->err = buf; else g_build_error = buf;
    return code;
}

int fm_dev_alloc(fm_matrix* m, void** p, size_t bytes)
{
    *p = nullptr;
    if (bytes == 0) bytes = 16;
    hipError_t e = hipMalloc(p, bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fm_fail(m, FM_ENOMEM, "hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
    }
    m->allocs.push_back(*p);
    return FM_OK;
}

void fm_dev_free(fm_matrix* m, void* p)
{
    if (p == nullptr) return;
    auto it = std::find(m->allocs.begin(), m->allocs.end(), p);
    if (it != m->allocs.end()) m->allocs.erase(it);
    (void)hipFree(p);
}

ProfScope::ProfScope(fm_matrix* m_, hipStream_t st_, int id_) : m(m_), st(st_), id(id_)
{
    if (!m->prof) return;
    for (hipEvent_t* ev : {&a, &b}) {
        if (!m->prof_pool.empty()) {
            *ev = m->prof_pool.back();
            m->prof_pool.pop_back();
        } else if (hipEventCreate(ev) != hipSuccess) {
            *ev = nullptr;
        }
    }
    if (a != nullptr) (void)hipEventRecord(a, st);
}

ProfScope::~ProfScope()
{
    if (!m->prof || a == nullptr || b == nullptr) return;
    (void)hipEventRecord(b, st);
    m->prof_recs.push_back({id, a, b});
}

static const char* const kKernelNames[FMK_COUNT] = {
    "rows_forward", "rows_refresh", "cols", "cols_long", "cols_tile", "cols_finish", "reduce", "bias"};

extern "C" int fm_profile_enable(fm_matrix* m, int32_t on)
{
    if (m == nullptr) return FM_EINVAL;
    m->prof = on != 0;
    return FM_OK;
}
extern "C" int fm_profile_kernels(void) { return FMK_COUNT; }
extern "C" const char* fm_profile_kernel_name(int32_t k) { return (k >= 0 && k < FMK_COUNT) ? kKernelNames[k] : ""; }

extern "C" int fm_profile_read(fm_matrix* m, int64_t* launches, double* total_ms)
{
    if (m == nullptr || launches == nullptr || total_ms == nullptr) return FM_EINVAL;
    FM_HIP(m, hipDeviceSynchronize());
    for (const ProfRec& r : m->prof_recs) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
            m->prof_launches[r.id] += 1;
            m->prof_ms[r.id] += (double)ms;
        }
        m->prof_pool.push_back(r.a);
        m->prof_pool.push_back(r.b);
    }
    m->prof_recs.clear();
    for (int k = 0; k < FMK_COUNT; ++k) {
        launches[k] = m->prof_launches[k];
        total_ms[k] = m->prof_ms[k];
        m->prof_launches[k] = 0;
        m->prof_ms[k] = 0.0;
    }
    return FM_OK;
}

extern "C" const char* fm_last_error(const fm_matrix* m) { return m != nullptr ? m->err.c_str() : g_build_error.c_str(); }

extern "C" int fm_destroy(fm_matrix* m)
{
    if (m == nullptr) return FM_OK;
    (void)hipDeviceSynchronize();
    fm_drop_graph(m);
    if (m->gstream != nullptr) (void)hipStreamDestroy(m->gstream);
    if (m->g_in != nullptr) (void)hipEventDestroy(m->g_in);
    if (m->g_out != nullptr) (void)hipEventDestroy(m->g_out);
    for (void* p : m->allocs) (void)hipFree(p);
    if (m->h_scal != nullptr) (void)hipHostFree(m->h_scal);
    if (m->side1 != nullptr) (void)hipStreamDestroy(m->side1);
    if (m->side2 != nullptr) (void)hipStreamDestroy(m->side2);
    for (hipEvent_t e : {m->ev_fork, m->ev_join1, m->ev_join2})
        if (e != nullptr) (void)hipEventDestroy(e);
    for (const ProfRec& r : m->prof_recs) {
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    for (hipEvent_t e : m->prof_pool) (void)hipEventDestroy(e);
    delete m;
    return FM_OK;
}

extern "C" int fm_build_csr(int64_t N, int64_t D, int64_t nnz, const int64_t* rowptr, const int32_t* col,
                            const float* val, void* hip_stream, fm_matrix** out)
{
    if (out == nullptr) return fm_fail(nullptr, FM_EINVAL, "out is NULL");
    *out = nullptr;
    if (N < 0 || D < 0 || nnz < 0 || rowptr == nullptr || (nnz > 0 && (col == nullptr || val == nullptr)))
        return fm_fail(nullptr, FM_EINVAL, "bad sizes or NULL arrays");
    if (N >= (1LL << 31) || D >= (1LL << 31) || nnz >= (1LL << 32))
        return fm_fail(nullptr, FM_ERANGE, "N, D must be < 2^31 and nnz < 2^32");
    if (rowptr[0] != 0 || rowptr[N] != nnz) return fm_fail(nullptr, FM_EUNSORTED, "rowptr[0] != 0 or rowptr[N] != nnz");
    for (int64_t i = 0; i < N; ++i) {
        const int64_t b = rowptr[i], e = rowptr[i + 1];
        if (e < b || e > nnz) return fm_fail(nullptr, FM_EUNSORTED, "rowptr not monotone at row %lld", (long long)i);
        for (int64_t t = b; t < e; ++t) {
            const int64_t c = col[t];
            if (c < 0 || c >= D)
                return fm_fail(nullptr, FM_ERANGE, "column %lld of row %lld outside [0,%lld)", (long long)c,
                               (long long)i, (long long)D);
            if (t > b && col[t - 1] >= c)
                return fm_fail(nullptr, FM_EUNSORTED, "columns of row %lld not strictly ascending", (long long)i);
        }
    }
    hipStream_t st = (hipStream_t)hip_stream;
    fm_matrix* m = new (std::nothrow) fm_matrix();
    if (m == nullptr) return fm_fail(nullptr, FM_ENOMEM, "out of host memory");
    m->N = N;
    m->D = D;
    m->nnz = nnz;
    int rc = FM_OK;
    auto up = [&](void** d, const void* h, size_t bytes) -> int {
        FM_TRY(fm_dev_alloc(m, d, bytes));
        if (bytes > 0) FM_HIP(m, hipMemcpyAsync(*d, h, bytes, hipMemcpyHostToDevice, st));
        return FM_OK;
    };
    rc = up((void**)&m->rowptr, rowptr, (size_t)(N + 1) * sizeof(int64_t));
    if (rc == FM_OK) rc = up((void**)&m->col, col, (size_t)nnz * sizeof(int32_t));
    if (rc == FM_OK) rc = up((void**)&m->val, val, (size_t)nnz * sizeof(float));
    if (rc == FM_OK) rc = fm_dev_alloc(m, (void**)&m->scal, (8 + FM_REDUCE_TMP) * sizeof(double));
    if (rc == FM_OK && hipHostMalloc((void**)&m->h_scal, 8 * sizeof(double)) != hipSuccess)
        rc = fm_fail(m, FM_ENOMEM, "pinned allocation failed");
    if (rc == FM_OK && hipStreamSynchronize(st) != hipSuccess) rc = fm_fail(m, FM_EHIP, "upload failed");
    if (rc == FM_OK) rc = fm_noalloc_init_device(m);  // set-up for fm_forward_noalloc on this device
    if (rc == FM_OK) rc = fm_dense_detect(m, st);
    if (rc != FM_OK) {
        g_build_error = m->err;
        fm_destroy(m);
        return rc;
    }
    *out = m;
    return FM_OK;
}

extern "C" int fm_get_csc(const fm_matrix* m, int64_t* colptr, int32_t* row, float* val)
{
    if (m == nullptr) return FM_EINVAL;
    fm_matrix* mm = const_cast<fm_matrix*>(m);
    if (!m->has_csc) return fm_fail(mm, FM_ESTATE, "CSC not built");
    FM_HIP(mm, hipDeviceSynchronize());
    if (colptr) FM_HIP(mm, hipMemcpy(colptr, m->colptr, (size_t)(m->D + 1) * sizeof(int64_t), hipMemcpyDeviceToHost));
    if (row && m->nnz) FM_HIP(mm, hipMemcpy(row, m->crow, (size_t)m->nnz * sizeof(int32_t), hipMemcpyDeviceToHost));
    if (val && m->nnz) FM_HIP(mm, hipMemcpy(val, m->cval, (size_t)m->nnz * sizeof(float), hipMemcpyDeviceToHost));
    return FM_OK;
}

extern "C" int fm_get_block_index(const fm_matrix* m, int64_t* row_bounds, int64_t* col_bounds, int64_t* cell_nnz)
{
    if (m == nullptr) return FM_EINVAL;
    fm_matrix* mm = const_cast<fm_matrix*>(m);
    if (m->P == 0) return fm_fail(mm, FM_ESTATE, "matrix not partitioned");
    if (col_bounds != nullptr && m->d_place != nullptr)
        return fm_fail(mm, FM_ESTATE, "the columns were placed one by one (fm_partition_placed): there are no column blocks");
    if (row_bounds) memcpy(row_bounds, m->h_rb.data(), (size_t)(m->P + 1) * sizeof(int64_t));
    if (col_bounds) memcpy(col_bounds, m->h_cb.data(), (size_t)(m->P + 1) * sizeof(int64_t));
    if (cell_nnz) {
        if (m->h_cell_nnz.empty()) return fm_fail(mm, FM_ESTATE, "the cell table is only kept for P <= %d", FM_MAXP_CELLS);
        memcpy(cell_nnz, m->h_cell_nnz.data(), (size_t)m->P * m->P * sizeof(int64_t));
    }
    return FM_OK;
}

extern "C" int fm_get_stratum_nnz(const fm_matrix* m, int32_t s, int64_t* nnz_out)
{
    if (m == nullptr || nnz_out == nullptr) return FM_EINVAL;
    fm_matrix* mm = const_cast<fm_matrix*>(m);
    if (m->P == 0) return fm_fail(mm, FM_ESTATE, "matrix not partitioned");
    if (s < 0 || s >= m->P) return fm_fail(mm, FM_EINVAL, "stratum %d outside [0,%d)", s, m->P);
    *nnz_out = m->h_strat_nnz_off[s + 1] - m->h_strat_nnz_off[s];
    return FM_OK;
}

// Pointer array over all nmaj rows (or columns) of one stratum or batch, expanded on the host from the list
// of the rows (columns) that have entries there: list positions [l0, l1), entries from ent0 on.
static int expand_ptr(fm_matrix* mm, const int32_t* nz_major, const int64_t* nz_beg, int64_t l0, int64_t l1,
                      int64_t ent0, int64_t ent1, int64_t nmaj, int64_t* ptr)
{
    const size_t cnt = (size_t)(l1 - l0);
    std::vector<int32_t> idx(cnt);
    std::vector<int64_t> beg(cnt);
    if (cnt > 0) {
        FM_HIP(mm, hipMemcpy(idx.data(), nz_major + l0, cnt * sizeof(int32_t), hipMemcpyDeviceToHost));
        FM_HIP(mm, hipMemcpy(beg.data(), nz_beg + l0, cnt * sizeof(int64_t), hipMemcpyDeviceToHost));
    }
    int64_t k = 0;
    for (size_t t = 0; t < cnt; ++t) {
        for (; k <= idx[t]; ++k) ptr[k] = beg[t] - ent0;  // rows up to and including this one start here
    }
    for (; k <= nmaj; ++k) ptr[k] = ent1 - ent0;
    return FM_OK;
}

static int get_stratum(const fm_matrix* m, int32_t s, bool by_rows, int64_t* ptr, int32_t* ind, float* val)
{
    if (m == nullptr) return FM_EINVAL;
    fm_matrix* mm = const_cast<fm_matrix*>(m);
    if (m->P == 0) return fm_fail(mm, FM_ESTATE, "matrix not partitioned");
    if (s < 0 || s >= m->P) return fm_fail(mm, FM_EINVAL, "stratum %d outside [0,%d)", s, m->P);
    FM_HIP(mm, hipDeviceSynchronize());
    const int64_t nmaj = by_rows ? m->N : m->D;
    const int64_t off = m->h_strat_nnz_off[s], cnt = m->h_strat_nnz_off[s + 1] - off;
    if (ptr) {
        const std::vector<int64_t>& lo = by_rows ? m->h_touch_off : m->h_ncol_off;
        FM_TRY(expand_ptr(mm, by_rows ? m->s_touched : m->s_ncol, by_rows ? m->s_touched_beg : m->s_ncol_beg, lo[s],
                          lo[s + 1], off, off + cnt, nmaj, ptr));
    }
    if (ind && cnt)
        FM_HIP(mm, hipMemcpy(ind, (by_rows ? m->s_col : m->s_row) + off, (size_t)cnt * sizeof(int32_t),
                             hipMemcpyDeviceToHost));
    if (val && cnt)
        FM_HIP(mm, hipMemcpy(val, (by_rows ? m->s_val : m->s_cval) + off, (size_t)cnt * sizeof(float),
                             hipMemcpyDeviceToHost));
    return FM_OK;
}

extern "C" int fm_get_stratum_csr(const fm_matrix* m, int32_t s, int64_t* rowptr, int32_t* col, float* val)
{
    return get_stratum(m, s, true, rowptr, col, val);
}
extern "C" int fm_get_stratum_csc(const fm_matrix* m, int32_t s, int64_t* colptr, int32_t* row, float* val)
{
    return get_stratum(m, s, false, colptr, row, val);
}

extern "C" int fm_get_batch_csc(const fm_matrix* m, int32_t b, int64_t* colptr, int32_t* row, float* val)
{
    if (m == nullptr) return FM_EINVAL;
    fm_matrix* mm = const_cast<fm_matrix*>(m);
    if (m->B == 0) return fm_fail(mm, FM_ESTATE, "row batches not built");
    if (b < 0 || b >= m->B) return fm_fail(mm, FM_EINVAL, "batch %d outside [0,%d)", b, m->B);
    FM_HIP(mm, hipDeviceSynchronize());
    const int64_t off = m->h_batch_nnz_off[b], cnt = m->h_batch_nnz_off[b + 1] - off;
    if (colptr)
        FM_TRY(expand_ptr(mm, m->b_ncol, m->b_ncol_beg, m->h_bcol_off[b], m->h_bcol_off[b + 1], off, off + cnt, m->D, colptr));
    if (row && cnt) FM_HIP(mm, hipMemcpy(row, m->b_row + off, (size_t)cnt * sizeof(int32_t), hipMemcpyDeviceToHost));
    if (val && cnt) FM_HIP(mm, hipMemcpy(val, m->b_cval + off, (size_t)cnt * sizeof(float), hipMemcpyDeviceToHost));
    return FM_OK;
}

// ------------------------------------------------------------ workspace ----

static int check_params(fm_matrix* m, const fm_params* p)
{
    if (p == nullptr) return fm_fail(m, FM_EINVAL, "params is NULL");
    int vec, lanes;
    if (!fm_shape_for_K(p->K, &vec, &lanes))
        return fm_fail(m, FM_EINVAL, "K=%d unsupported (1..64, or a multiple of 4 up to 256)", p->K);
    if (p->loss != FM_LOSS_SQUARED && p->loss != FM_LOSS_LOGISTIC) return fm_fail(m, FM_EINVAL, "unknown loss %d", p->loss);
    if (p->half_gather && p->K % 4 != 0) return fm_fail(m, FM_EINVAL, "half_gather needs K to be a multiple of 4");
    return FM_OK;
}

// stratified calls keep fp32 gathers: their incremental refresh adds fp32 changes to aggregates that
// would have been formed from rounded factors
static int no_half(fm_matrix* m, const fm_params* p)
{
    if (p->half_gather) return fm_fail(m, FM_EINVAL, "half_gather applies to fm_forward, fm_evaluate, fm_sgd_epoch and fm_minibatch_epoch");
    return FM_OK;
}

// Packed rows are used when [G | r] of a row fits one 128-byte line (a whole number of float4,
// K <= 28): a column-side gather is then a single request.  For larger K a row of G is one or
// more whole lines by itself and the planar layout gathers fewer of them.  The option aux_planar
// selects the planar layout always.
bool fm_aux_packed(const fm_matrix* m, int32_t K) { return !m->opt.aux_planar && K % 4 == 0 && K + 1 <= 32; }

static int64_t packed_stride(int32_t K) { return ((int64_t)K + 3 + 15) / 16 * 16; }

int fm_cols_packed_mode(const fm_matrix* m, int32_t K) { return fm_aux_packed(m, K) ? FM_PACKED_LANE : FM_PLANAR; }

int64_t fm_aux_floats(const fm_matrix* m, int32_t K)
{
    return fm_aux_packed(m, K) ? m->N * packed_stride(K) : m->N * ((int64_t)K + 3);
}

FmAux fm_aux_layout(const fm_matrix* m, int32_t K)
{
    FmAux x;
    if (fm_aux_packed(m, K)) {
        x.gs = x.ss = packed_stride(K);
        x.G = m->aux;
        x.r = m->aux + K;
        x.a = m->aux + K + 1;
        x.q = m->aux + K + 2;
    } else {
        x.gs = K;
        x.ss = 1;
        x.G = m->aux;
        x.r = m->aux + m->N * (int64_t)K;
        x.a = x.r + m->N;
        x.q = x.a + m->N;
    }
    return x;
}

bool fm_side_streams(fm_matrix* m)
{
    if (!m->opt.side_streams) return false;
    if (m->side_state == 0) {
        m->side_state = -1;
        if (hipStreamCreateWithFlags(&m->side1, hipStreamNonBlocking) == hipSuccess &&
            hipStreamCreateWithFlags(&m->side2, hipStreamNonBlocking) == hipSuccess &&
            hipEventCreateWithFlags(&m->ev_fork, hipEventDisableTiming) == hipSuccess &&
            hipEventCreateWithFlags(&m->ev_join1, hipEventDisableTiming) == hipSuccess &&
            hipEventCreateWithFlags(&m->ev_join2, hipEventDisableTiming) == hipSuccess)
            m->side_state = 1;
        else
            (void)hipGetLastError();
    }
    return m->side_state == 1;
}

void fm_drop_graph(fm_matrix* m)
{
    if (m->gexec != nullptr) {
        (void)hipGraphExecDestroy(m->gexec);
        m->gexec = nullptr;
    }
}

void fm_drop_workspace(fm_matrix* m)
{
    fm_drop_graph(m);
    for (void* p : {(void*)m->aux, (void*)m->dV, (void*)m->dwn, (void*)m->part, (void*)m->row_part})
        fm_dev_free(m, p);
    m->aux = m->dV = m->part = m->row_part = nullptr;
    m->dwn = nullptr;
    m->wsK = 0;
    m->aux_full = false;
    m->aux_held = false;
}

// (re)allocate the per-K workspace
static int ensure_ws(fm_matrix* m, int32_t K)
{
    if (m->wsK == K) return FM_OK;
    fm_drop_workspace(m);
    if (m->has_csc) {  // the LDS tiles of the dense-ish columns are shaped for K
        int shape[3];
        fm_tile_shape(m, K, &shape[0], &shape[1], &shape[2]);
        if (memcmp(shape, m->lfull_shape, sizeof(shape)) != 0) {
            FM_HIP(m, hipDeviceSynchronize());
            FM_TRY(fm_build_full_index(m, K, nullptr));
            FM_HIP(m, hipDeviceSynchronize());
        }
    }
    const size_t D = (size_t)m->D;
    FM_TRY(fm_dev_alloc(m, (void**)&m->aux, (size_t)std::max<int64_t>(fm_aux_floats(m, K), 1) * sizeof(float)));
    const int64_t items = std::max<int64_t>(std::max<int64_t>(m->lfull.nitems, m->lstrat.nitems),
                                            std::max<int64_t>(m->lbatch.nitems, m->ldense.nitems));
    FM_TRY(fm_dev_alloc(m, (void**)&m->part,
                        (size_t)std::max<int64_t>(items, 1) * (size_t)fm_part_stride(K) * sizeof(float)));
    FM_TRY(fm_dev_alloc(m, (void**)&m->row_part, (size_t)std::max<int64_t>(fm_rows_grid(m->N, K), 1) * 2 * sizeof(float)));
    if (m->P > 0) {
        FM_TRY(fm_dev_alloc(m, (void**)&m->dV, D * K * sizeof(float)));
        FM_TRY(fm_dev_alloc(m, (void**)&m->dwn, D * sizeof(float2)));
    }
    m->wsK = K;
    return FM_OK;
}

static int ensure_strat_ws(fm_matrix* m, int32_t K)
{
    return ensure_ws(m, K);  // fm_partition dropped any older workspace, so dV/dwn are there
}

static void fill_long(const fm_matrix* m, ColArgs& A, const LongIndex& li, int32_t s, bool strat)
{
    const int64_t l0 = strat ? li.h_long_off[s] : 0, l1 = strat ? li.h_long_off[s + 1] : li.nlong;
    const int64_t i0 = strat ? li.h_item_off[s] : 0, i1 = strat ? li.h_item_off[s + 1] : li.nitems;
    A.nlong = l1 - l0;
    A.nitems = i1 - i0;
    A.long_base = l0;
    A.item_base = i0;
    A.long_col = li.long_col;
    A.long_first = li.long_first;
    A.item_col = li.item_col;
    A.item_beg = li.item_beg;
    A.item_len = li.item_len;
    A.order = strat ? nullptr : li.order;
    A.ord_beg = li.ord_beg;
    A.ord_len = li.ord_len;
    for (int x = 0; x <= FM_XCDS; ++x) A.list_off[x] = li.list_off[x];
    for (int x = 0; x < FM_XCDS; ++x) A.list_mid[x] = li.list_mid[x];
    A.tile_rows = li.tile_rows;
    A.ntiles = strat ? 0 : li.ntiles;
    A.tile_ptr = li.tile_ptr;
    A.lin_mode = 0;
    A.vlong = strat ? nullptr : li.vlong;
    A.nvlong = strat ? 0 : li.nvlong;
    A.vlong_items = m->tune.vlong;
    const int64_t s0 = strat ? li.h_short_off[s] : 0, s1 = strat ? li.h_short_off[s + 1] : li.nshort;
    A.short_col = li.short_col != nullptr ? li.short_col + s0 : nullptr;
    A.short_beg = li.short_beg != nullptr ? li.short_beg + s0 : nullptr;
    A.short_len = li.short_len != nullptr ? li.short_len + s0 : nullptr;
    A.nshort = s1 - s0;
}

// RowArgs outputs pointing into the handle's aggregate rows [G | r | a | q | pad]
static void aux_outputs(fm_matrix* m, int32_t K, RowArgs& A, bool with_aq)
{
    const FmAux x = fm_aux_layout(m, K);
    A.whole_rows = (fm_aux_packed(m, K) && A.y != nullptr) ? 1 : 0;  // never leave a line partly written
    A.G = x.G;
    A.gs = x.gs;
    A.ss = x.ss;
    A.r = x.r;
    A.a = with_aq ? x.a : nullptr;
    A.q = with_aq ? x.q : nullptr;
}

// ---------------------------------------------------------------- forward ----

// With half_gather: refresh the handle's half-precision copy of V (one streaming pass) and hand it to the row kernel.
static int half_copy(fm_matrix* m, const fm_params* p, const float* V, const _Float16** out, hipStream_t st)
{
    *out = nullptr;
    if (!p->half_gather) return FM_OK;
    const int64_t n = m->D * (int64_t)p->K;
    if (m->Vh == nullptr || m->VhK != p->K) {
        if (m->Vh != nullptr) {
            FM_HIP(m, hipDeviceSynchronize());
            fm_dev_free(m, m->Vh);
            m->Vh = nullptr;
        }
        FM_TRY(fm_dev_alloc(m, (void**)&m->Vh, (size_t)std::max<int64_t>(n, 1) * sizeof(_Float16)));
        m->VhK = p->K;
    }
    FM_TRY(fm_to_half(m, V, m->Vh, n, st));
    *out = m->Vh;
    return FM_OK;
}

// mode 0: caller arrays (dense); 1: handle's aggregate rows, G and r; 2: handle's rows, G r a q
static int run_forward(fm_matrix* m, const fm_params* p, const float* y, const float* w0, const float* w,
                       const float* V, float* yhat, float* a, float* G, float* q, float* r, int mode, bool want_sums,
                       hipStream_t st)
{
    RowArgs A;
    memset(&A, 0, sizeof(A));
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
    if (mode == 0) {
        A.a = a;
        A.G = G;
        A.q = q;
        A.r = r;
        A.gs = p->K;
        A.ss = 1;
    } else {
        aux_outputs(m, p->K, A, mode == 2);
        m->aux_held = true;
    }
    A.row_part = (want_sums && y != nullptr) ? m->row_part : nullptr;
    A.loss = p->loss;
    A.s = p->loss_scale;
    FM_TRY(half_copy(m, p, V, &A.Vh, st));
    const bool dense = A.Vh == nullptr && fm_dense_shape_ok(m, p->K);
    if (dense) A.dense_D = (int32_t)m->D;
    FM_TRY(fm_launch_rows(m, A, false, st));
    // one (loss, multiplier) pair per row block of the sparse kernel, per 32 rows of the dense one
    const int64_t pairs = dense ? (m->N + 31) / 32 : fm_rows_grid(m->N, p->K);
    if (A.row_part != nullptr) FM_TRY(fm_reduce_pairs(m, m->row_part, pairs, m->scal + 0, st));
    return FM_OK;
}

extern "C" int fm_forward(fm_matrix* m, const fm_params* p, const float* y, const float* w0, const float* w,
                          const float* V, float* yhat, float* a, float* G, float* q, float* r, double* loss_sum,
                          void* hip_stream)
{
    if (m == nullptr) return FM_EINVAL;
    FM_TRY(check_params(m, p));
    if (w0 == nullptr || w == nullptr || V == nullptr) return fm_fail(m, FM_EINVAL, "w0, w, V must not be NULL");
    if ((r != nullptr || loss_sum != nullptr) && y == nullptr) return fm_fail(m, FM_EINVAL, "r and loss_sum need y");
    FM_TRY(fm_check_vec_aligned(m, {V, G}));
    hipStream_t st = (hipStream_t)hip_stream;
    FM_TRY(ensure_ws(m, p->K));
    if (m->N == 0) {
        if (loss_sum) *loss_sum = 0.0;
        return FM_OK;
    }
    FM_TRY(run_forward(m, p, y, w0, w, V, yhat, a, G, q, r, 0, loss_sum != nullptr, st));
    if (loss_sum != nullptr) {
        FM_HIP(m, hipMemcpyAsync(m->h_scal, m->scal, 2 * sizeof(double), hipMemcpyDeviceToHost, st));
        FM_HIP(m, hipStreamSynchronize(st));
        *loss_sum = m->h_scal[0];
    }
    return FM_OK;
}

extern "C" int fm_evaluate(fm_matrix* m, const fm_params* p, const float* y, const float* w0, const float* w,
                           const float* V, double* metrics, void* hip_stream)
{
    if (m == nullptr) return FM_EINVAL;
    FM_TRY(check_params(m, p));
    if (y == nullptr || w0 == nullptr || w == nullptr || V == nullptr || metrics == nullptr)
        return fm_fail(m, FM_EINVAL, "y, w0, w, V, metrics must not be NULL");
    FM_TRY(fm_check_vec_aligned(m, {V}));
    hipStream_t st = (hipStream_t)hip_stream;
    FM_TRY(ensure_ws(m, p->K));
    metrics[0] = metrics[1] = metrics[2] = 0.0;
    if (m->N == 0) return FM_OK;
    // the scores go to the start of the aggregate storage, which holds nothing afterwards
    m->aux_held = false;
    m->aux_full = false;
    RowArgs A;
    memset(&A, 0, sizeof(A));
    A.N = m->N;
    A.K = p->K;
    A.rowptr = m->rowptr;
    A.col = m->col;
    A.val = m->val;
    A.w0 = w0;
    A.w = w;
    A.V = V;
    A.y = y;
    A.yhat = m->aux;
    A.gs = p->K;
    A.ss = 1;
    A.row_part = m->row_part;
    A.loss = p->loss;
    A.s = 1.f;
    FM_TRY(half_copy(m, p, V, &A.Vh, st));
    const bool dense = A.Vh == nullptr && fm_dense_shape_ok(m, p->K);
    if (dense) A.dense_D = (int32_t)m->D;
    FM_TRY(fm_launch_rows(m, A, false, st));
    FM_TRY(fm_reduce_pairs(m, m->row_part, dense ? (m->N + 31) / 32 : fm_rows_grid(m->N, p->K), m->scal + 0, st));
    FM_TRY(fm_reduce_eval(m, m->aux, y, m->N, 0, m->scal + 4, st));
    FM_TRY(fm_reduce_eval(m, m->aux, y, m->N, 1, m->scal + 5, st));
    FM_HIP(m, hipMemcpyAsync(m->h_scal, m->scal, 6 * sizeof(double), hipMemcpyDeviceToHost, st));
    FM_HIP(m, hipStreamSynchronize(st));
    const double n = (double)m->N;
    metrics[0] = m->h_scal[0] / n;
    metrics[1] = sqrt(m->h_scal[4] / n);
    metrics[2] = m->h_scal[5] / n;
    return FM_OK;
}

// --------------------------------------------------------------- gradient ----

// Work decomposition of a column pass over the whole matrix: the items of the CSC copy, or, for a matrix that
// stores every column in every row, chunks of rows of the dense matrix.
static void full_long(fm_matrix* m, const fm_params* p, ColArgs& A)
{
    if (fm_dense_shape_ok(m, p->K) && m->ldense.long_col != nullptr) {
        fill_long(m, A, m->ldense, 0, false);
        A.X = m->val;
        A.chunk_rows = m->dense_chunk_rows;
        A.nchunks = m->dense_chunks;
    } else {
        fill_long(m, A, m->lfull, 0, false);
    }
}

static void base_col_args(fm_matrix* m, const fm_params* p, ColArgs& A)
{
    memset(&A, 0, sizeof(A));
    A.D = m->D;
    A.K = p->K;
    A.lambda_w = p->lambda_w;
    A.lambda_v = p->lambda_v;
    A.eta = p->eta;
    A.N = m->N;
    A.part = m->part;
    A.ps = fm_part_stride(p->K);
}

extern "C" int fm_gradient(fm_matrix* m, const fm_params* p, const float* r, const float* G, const float* w,
                           const float* V, float* grad_w0, float* grad_w, float* grad_V, void* hip_stream)
{
    if (m == nullptr) return FM_EINVAL;
    FM_TRY(check_params(m, p));
    if (!m->has_csc) return fm_fail(m, FM_ESTATE, "fm_gradient needs fm_build_csc first");
    if (r == nullptr || G == nullptr || w == nullptr || V == nullptr)
        return fm_fail(m, FM_EINVAL, "r, G, w, V must not be NULL");
    FM_TRY(fm_check_vec_aligned(m, {G, V, grad_V}));
    hipStream_t st = (hipStream_t)hip_stream;
    FM_TRY(ensure_ws(m, p->K));
    if (grad_w0 != nullptr) {
        FM_TRY(fm_reduce_sum(m, r, m->N, 1, false, m->scal + 1, st));
        FM_TRY(fm_bias_step(m, nullptr, m->scal + 1, 0.f, grad_w0, st));
    }
    if (m->D == 0 || (grad_w == nullptr && grad_V == nullptr)) return FM_OK;
    ColArgs A;
    base_col_args(m, p, A);
    A.ptr = m->colptr;
    A.row = m->crow;
    A.val = m->cval;
    if (fm_aux_packed(m, p->K)) {
        // one streaming pass puts r and G into packed aggregate rows, so that every gather of the
        // column pass is one request (and dense-ish columns can be staged through LDS)
        FM_TRY(fm_pack_aux(m, r, G, st));
        m->aux_held = true;
        m->aux_full = false;
        const FmAux x = fm_aux_layout(m, p->K);
        A.r = x.r;
        A.G = x.G;
        A.gs = x.gs;
        A.rs = x.ss;
        A.packed = fm_cols_packed_mode(m, p->K);
    } else {
        A.r = r;
        A.G = G;
        A.gs = p->K;
        A.rs = 1;
    }
    A.w = const_cast<float*>(w);
    A.V = const_cast<float*>(V);
    A.grad_w = grad_w;
    A.grad_V = grad_V;
    full_long(m, p, A);
    return fm_launch_cols(m, A, false, st);
}

// ------------------------------------------------------------ full epoch ----

extern "C" int fm_sgd_epoch(fm_matrix* m, const fm_params* p, const float* y, float* w0, float* w, float* V,
                            double* objective, void* hip_stream)
{
    if (m == nullptr) return FM_EINVAL;
    FM_TRY(check_params(m, p));
    if (!m->has_csc) return fm_fail(m, FM_ESTATE, "fm_sgd_epoch needs fm_build_csc first");
    if (y == nullptr || w0 == nullptr || w == nullptr || V == nullptr)
        return fm_fail(m, FM_EINVAL, "y, w0, w, V must not be NULL");
    FM_TRY(fm_check_vec_aligned(m, {V}));
    hipStream_t st = (hipStream_t)hip_stream;
    FM_TRY(ensure_ws(m, p->K));
    if (m->N == 0 || m->D == 0) {
        if (objective) objective[0] = objective[1] = 0.0;
        return FM_OK;
    }
    // steps 1-3: G, r, loss and sum r
    FM_TRY(run_forward(m, p, y, w0, w, V, nullptr, nullptr, nullptr, nullptr, nullptr, 1, true, st));
    m->aux_full = false;
    if (objective != nullptr) {  // regulariser at the parameters the epoch starts from
        FM_TRY(fm_reduce_sum(m, w, m->D, 1, true, m->scal + 2, st));
        FM_TRY(fm_reduce_sum(m, V, m->D * (int64_t)p->K, 1, true, m->scal + 3, st));
    }
    // steps 4-5 fused: gradient of every column and the step on w, V
    ColArgs A;
    base_col_args(m, p, A);
    A.ptr = m->colptr;
    A.row = m->crow;
    A.val = m->cval;
    const FmAux x = fm_aux_layout(m, p->K);
    A.r = x.r;
    A.G = x.G;
    A.gs = x.gs;
    A.rs = x.ss;
    A.packed = fm_cols_packed_mode(m, p->K);
    A.w = w;
    A.V = V;
    full_long(m, p, A);
    FM_TRY(fm_launch_cols(m, A, true, st));
    if (p->update_w0) FM_TRY(fm_bias_step(m, w0, m->scal + 1, p->eta, nullptr, st));
    if (objective != nullptr) {
        FM_HIP(m, hipMemcpyAsync(m->h_scal, m->scal, 4 * sizeof(double), hipMemcpyDeviceToHost, st));
        FM_HIP(m, hipStreamSynchronize(st));
        objective[0] = (double)p->loss_scale * m->h_scal[0];
        objective[1] = 0.5 * (double)p->lambda_w * m->h_scal[2] + 0.5 * (double)p->lambda_v * m->h_scal[3];
    }
    return FM_OK;
}

// ------------------------------------------------------- stratified epoch ----

extern "C" int fm_stratified_begin(fm_matrix* m, const fm_params* p, const float* y, const float* w0,
                                   const float* w, const float* V, void* hip_stream)
{
    if (m == nullptr) return FM_EINVAL;
    FM_TRY(check_params(m, p));
    FM_TRY(no_half(m, p));
    if (m->P == 0) return fm_fail(m, FM_ESTATE, "stratified calls need fm_partition first");
    if (y == nullptr || w0 == nullptr || w == nullptr || V == nullptr)
        return fm_fail(m, FM_EINVAL, "y, w0, w, V must not be NULL");
    FM_TRY(fm_check_vec_aligned(m, {V}));
    hipStream_t st = (hipStream_t)hip_stream;
    FM_TRY(ensure_strat_ws(m, p->K));
    FM_TRY(run_forward(m, p, y, w0, w, V, nullptr, nullptr, nullptr, nullptr, nullptr, 2, false, st));
    m->aux_full = true;
    return FM_OK;
}

// Regulariser shares of P floor-split row blocks: the table, the bounds, and the two values it holds.
static void set_shares(ColArgs& A, const float* rho, const int64_t* bounds, int64_t N, int32_t P)
{
    A.rho = rho;
    A.rb = bounds;
    const int64_t base = N / P;
    A.rho_small = (float)((double)base / (double)N);
    A.rho_big = (float)((double)(base + 1) / (double)N);
}

// Column-side arguments of stratum s (s == P: the flush after the last stratum).
static void strat_col_args(fm_matrix* m, const fm_params* p, int32_t s, float* w, float* V, bool lazy, ColArgs& A)
{
    base_col_args(m, p, A);
    A.w = w;
    A.V = V;
    A.P = m->P;
    A.s = s;
    if (!p->reg_full_per_cell) set_shares(A, m->d_rho, m->d_rb, m->N, m->P);
    A.place = m->d_place;
    if (lazy) A.lazy_last = m->lazy_last;
}

// One stratum.  lazy: columns that are empty in their cell postpone their regulariser-only step
// (the caller starts the epoch with lazy_last = 0 and flushes after the last stratum).
static int stratified_step(fm_matrix* m, const fm_params* p, int32_t s, const float* y, const float* w0, float* w,
                           float* V, bool lazy, hipStream_t st)
{
    // phase A: block gradients of the stratum's P cells and the step on every column block
    ColArgs A;
    strat_col_args(m, p, s, w, V, lazy, A);
    A.ptr = nullptr;  // no pointer array per stratum: short columns carry their extent, long ones their items
    A.mark = lazy ? nullptr : m->col_mark;
    A.row = m->s_row;
    A.val = m->s_cval;
    const FmAux x = fm_aux_layout(m, p->K);
    A.r = x.r;
    A.G = x.G;
    A.gs = x.gs;
    A.rs = x.ss;
    A.packed = fm_cols_packed_mode(m, p->K);
    if (!p->stale_aux) {  // the changes are only recorded for the refresh
        A.dV = m->dV;
        A.dwn = m->dwn;
    }
    fill_long(m, A, m->lstrat, s, true);
    FM_TRY(fm_launch_cols(m, A, true, st));
    if (p->stale_aux) return FM_OK;  // Algorithm 1: the aggregates wait for the re-computation
    // phase B: incremental refresh of the aggregates and multipliers
    RowArgs R;
    memset(&R, 0, sizeof(R));
    R.N = m->N;
    R.K = p->K;
    if (p->refresh_all_rows) {
        R.rowptr = m->rowptr;
        R.col = m->col;
        R.val = m->val;
    } else {
        R.col = m->s_col;
        R.val = m->s_val;
        // only the rows that have an entry in this stratum
        R.rows = m->s_touched + m->h_touch_off[s];
        R.rowptr = m->s_touched_beg + m->h_touch_off[s];
        R.N = m->h_touch_off[s + 1] - m->h_touch_off[s];
    }
    R.w0 = w0;
    R.V = m->dV;
    R.dwn = m->dwn;
    R.y = y;
    aux_outputs(m, p->K, R, true);
    R.loss = p->loss;
    R.s = p->loss_scale;
    return fm_launch_rows(m, R, true, st);
}

extern "C" int fm_stratified_step(fm_matrix* m, const fm_params* p, int32_t s, const float* y, const float* w0,
                                  float* w, float* V, void* hip_stream)
{
    if (m == nullptr) return FM_EINVAL;
    FM_TRY(check_params(m, p));
    FM_TRY(no_half(m, p));
    if (m->P == 0) return fm_fail(m, FM_ESTATE, "stratified calls need fm_partition first");
    if (s < 0 || s >= m->P) return fm_fail(m, FM_EINVAL, "stratum %d outside [0,%d)", s, m->P);
    if (y == nullptr || w0 == nullptr || w == nullptr || V == nullptr)
        return fm_fail(m, FM_EINVAL, "y, w0, w, V must not be NULL");
    FM_TRY(fm_check_vec_aligned(m, {V}));
    if (m->wsK != p->K || !m->aux_full) return fm_fail(m, FM_ESTATE, "call fm_stratified_begin first");
    return stratified_step(m, p, s, y, w0, w, V, false, (hipStream_t)hip_stream);
}

extern "C" int fm_stratified_end(fm_matrix* m, const fm_params* p, float* w0, void* hip_stream)
{
    if (m == nullptr) return FM_EINVAL;
    FM_TRY(check_params(m, p));
    if (m->wsK != p->K || !m->aux_full) return fm_fail(m, FM_ESTATE, "call fm_stratified_begin first");
    if (w0 == nullptr) return fm_fail(m, FM_EINVAL, "w0 must not be NULL");
    hipStream_t st = (hipStream_t)hip_stream;
    if (p->update_w0) {
        const FmAux x = fm_aux_layout(m, p->K);
        FM_TRY(fm_reduce_sum(m, x.r, m->N, x.ss, false, m->scal + 1, st));
        FM_TRY(fm_bias_step(m, w0, m->scal + 1, p->eta, nullptr, st));
    }
    return FM_OK;
}

// Everything one stratified epoch enqueues (no allocation, no host transfer, no wait).
static int enqueue_stratified_epoch(fm_matrix* m, const fm_params* p, const float* y, float* w0, float* w, float* V,
                                    bool lazy, hipStream_t st)
{
    FM_TRY(run_forward(m, p, y, w0, w, V, nullptr, nullptr, nullptr, nullptr, nullptr, 2, false, st));
    if (lazy) FM_TRY(fm_fill_i32(m, m->lazy_last, m->D, 0, st));
    for (int32_t s = 0; s < m->P; ++s) FM_TRY(stratified_step(m, p, s, y, w0, w, V, lazy, st));
    if (lazy) {
        ColArgs F;
        strat_col_args(m, p, m->P, w, V, true, F);
        FM_TRY(fm_launch_cols_flush(m, F, st));
    }
    if (p->update_w0) {
        const FmAux x = fm_aux_layout(m, p->K);
        FM_TRY(fm_reduce_sum(m, x.r, m->N, x.ss, false, m->scal + 1, st));
        FM_TRY(fm_bias_step(m, w0, m->scal + 1, p->eta, nullptr, st));
    }
    return FM_OK;
}

static bool graph_ready(fm_matrix* m)
{
    if (m->graph_state == 0) {
        m->graph_state = -1;
        if (hipStreamCreateWithFlags(&m->gstream, hipStreamNonBlocking) == hipSuccess &&
            hipEventCreateWithFlags(&m->g_in, hipEventDisableTiming) == hipSuccess &&
            hipEventCreateWithFlags(&m->g_out, hipEventDisableTiming) == hipSuccess)
            m->graph_state = 1;
        else
            (void)hipGetLastError();
    }
    return m->graph_state == 1;
}

// Capture the epoch on the internal stream (or reuse the capture made for the same arguments) and
// replay it between two events on the caller's stream.  Returns FM_ESTATE if no graph could be
// built: the caller then enqueues the epoch directly.
static int replay_stratified_epoch(fm_matrix* m, const fm_params* p, const float* y, float* w0, float* w, float* V,
                                   bool lazy, hipStream_t st)
{
    const void* key[4] = {y, w0, w, V};
    const bool same = m->gexec != nullptr && memcmp(&m->gkey_p, p, sizeof(fm_params)) == 0 &&
                      memcmp(m->gkey_ptr, key, sizeof(key)) == 0 && m->gkey_lazy == lazy;
    if (!same) {
        fm_drop_graph(m);
        (void)fm_side_streams(m);  // created outside the capture
        if (hipStreamBeginCapture(m->gstream, hipStreamCaptureModeThreadLocal) != hipSuccess) {
            (void)hipGetLastError();
            return FM_ESTATE;
        }
        const int rc = enqueue_stratified_epoch(m, p, y, w0, w, V, lazy, m->gstream);
        hipGraph_t graph = nullptr;
        const hipError_t e = hipStreamEndCapture(m->gstream, &graph);
        if (rc != FM_OK || e != hipSuccess || graph == nullptr) {
            (void)hipGetLastError();
            if (graph != nullptr) (void)hipGraphDestroy(graph);
            return FM_ESTATE;
        }
        const hipError_t ei = hipGraphInstantiate(&m->gexec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        if (ei != hipSuccess) {
            (void)hipGetLastError();
            m->gexec = nullptr;
            return FM_ESTATE;
        }
        m->gkey_p = *p;
        memcpy(m->gkey_ptr, key, sizeof(key));
        m->gkey_lazy = lazy;
    }
    FM_HIP(m, hipEventRecord(m->g_in, st));
    FM_HIP(m, hipStreamWaitEvent(m->gstream, m->g_in, 0));
    FM_HIP(m, hipGraphLaunch(m->gexec, m->gstream));
    FM_HIP(m, hipEventRecord(m->g_out, m->gstream));
    FM_HIP(m, hipStreamWaitEvent(st, m->g_out, 0));
    return FM_OK;
}

extern "C" int fm_stratified_epoch(fm_matrix* m, const fm_params* p, const float* y, float* w0, float* w, float* V,
                                   double* objective, void* hip_stream)
{
    if (m == nullptr) return FM_EINVAL;
    FM_TRY(check_params(m, p));
    FM_TRY(no_half(m, p));
    if (m->P == 0) return fm_fail(m, FM_ESTATE, "stratified calls need fm_partition first");
    if (y == nullptr || w0 == nullptr || w == nullptr || V == nullptr)
        return fm_fail(m, FM_EINVAL, "y, w0, w, V must not be NULL");
    FM_TRY(fm_check_vec_aligned(m, {V}));
    hipStream_t st = (hipStream_t)hip_stream;
    FM_TRY(ensure_strat_ws(m, p->K));
    // The refresh of a stratum reads the change of a column only where the column has entries in
    // its cell, so the regulariser-only steps of the other columns can wait (not when every row
    // is refreshed from every column's change).
    const bool lazy = (!p->refresh_all_rows || p->stale_aux) && m->lazy_last != nullptr && m->opt.lazy_reg;
    // small strata are bound by their launches: replay them from a graph
    const int gmode = m->opt.graph;  // 0 never, 1 for matrices whose strata are small enough for the launches to dominate, 2 always
    // (worth it from some tens of launches on: below that the two events and the graph launch cost more; with
    // 32 strata or more the replay pays even when the strata are large: 2 % on the click-style and the hashed workload)
    const bool small = m->P >= 32 || (m->nnz / m->P < (int64_t(1) << 20) && m->P >= 16);
    bool done = false;
    if (!m->prof && (gmode == 2 || (gmode == 1 && small)) && graph_ready(m)) {
        const int rc = replay_stratified_epoch(m, p, y, w0, w, V, lazy, st);
        if (rc == FM_OK)
            done = true;
        else if (rc != FM_ESTATE)
            return rc;
    }
    if (!done) FM_TRY(enqueue_stratified_epoch(m, p, y, w0, w, V, lazy, st));
    m->aux_full = true;
    m->aux_held = true;
    if (objective != nullptr) {
        FM_TRY(run_forward(m, p, y, w0, w, V, nullptr, nullptr, nullptr, nullptr, nullptr, 2, true, st));
        FM_TRY(fm_reduce_sum(m, w, m->D, 1, true, m->scal + 2, st));
        FM_TRY(fm_reduce_sum(m, V, m->D * (int64_t)p->K, 1, true, m->scal + 3, st));
        FM_HIP(m, hipMemcpyAsync(m->h_scal, m->scal, 4 * sizeof(double), hipMemcpyDeviceToHost, st));
        FM_HIP(m, hipStreamSynchronize(st));
        objective[0] = (double)p->loss_scale * m->h_scal[0];
        objective[1] = 0.5 * (double)p->lambda_w * m->h_scal[2] + 0.5 * (double)p->lambda_v * m->h_scal[3];
    }
    return FM_OK;
}

// ------------------------------------------------------- mini-batch epoch ----

extern "C" int fm_minibatch_epoch(fm_matrix* m, const fm_params* p, const float* y, float* w0, float* w, float* V,
                                  double* objective, void* hip_stream)
{
    if (m == nullptr) return FM_EINVAL;
    FM_TRY(check_params(m, p));
    if (m->B == 0) return fm_fail(m, FM_ESTATE, "fm_minibatch_epoch needs fm_partition_batches first");
    if (y == nullptr || w0 == nullptr || w == nullptr || V == nullptr)
        return fm_fail(m, FM_EINVAL, "y, w0, w, V must not be NULL");
    FM_TRY(fm_check_vec_aligned(m, {V}));
    hipStream_t st = (hipStream_t)hip_stream;
    FM_TRY(ensure_ws(m, p->K));
    m->aux_full = false;
    m->aux_held = true;
    const FmAux x = fm_aux_layout(m, p->K);
    // a column without entries in a batch only takes the regulariser's step there: postponed
    // until the column next has entries, or the epoch ends
    const bool lazy = m->opt.lazy_reg;
    if (lazy) FM_TRY(fm_fill_i32(m, m->lazy_last, m->D, 0, st));
    auto col_args = [&](int32_t b, ColArgs& A) {
        base_col_args(m, p, A);
        A.w = w;
        A.V = V;
        A.P = m->B;
        A.s = b;
        A.batch = 1;
        if (!p->reg_full_per_cell) set_shares(A, m->d_brho, m->d_bb, m->N, m->B);
        if (lazy) A.lazy_last = m->lazy_last;
    };
    for (int32_t b = 0; b < m->B; ++b) {
        const int64_t r0 = m->h_bb[b], nb = m->h_bb[b + 1] - r0;
        if (nb > 0) {  // steps 1-3 on the rows of the batch, at the parameters as they stand
            RowArgs R;
            memset(&R, 0, sizeof(R));
            R.N = nb;
            R.K = p->K;
            R.rowptr = m->rowptr + r0;
            R.col = m->col;
            R.val = m->val;
            R.w0 = w0;
            R.w = w;
            R.V = V;
            R.y = y + r0;
            R.G = x.G + r0 * x.gs;
            R.gs = x.gs;
            R.ss = x.ss;
            R.r = x.r + r0 * x.ss;
            R.whole_rows = fm_aux_packed(m, p->K) ? 1 : 0;
            R.row_part = p->update_w0 ? m->row_part : nullptr;
            R.loss = p->loss;
            R.s = p->loss_scale;
            FM_TRY(half_copy(m, p, V, &R.Vh, st));  // the factors as they stand
            FM_TRY(fm_launch_rows(m, R, false, st));
            if (R.row_part != nullptr)
                FM_TRY(fm_reduce_pairs(m, m->row_part, fm_rows_grid(nb, p->K), m->scal + 0, st));
        }
        // steps 4-5 over the batch's rows: gradient and step of every column that has entries there
        ColArgs A;
        col_args(b, A);
        A.ptr = nullptr;
        A.mark = lazy ? nullptr : m->col_mark;
        A.row = m->b_row;
        A.val = m->b_cval;
        A.r = x.r;
        A.G = x.G;
        A.gs = x.gs;
        A.rs = x.ss;
        A.packed = fm_cols_packed_mode(m, p->K);
        fill_long(m, A, m->lbatch, b, true);
        FM_TRY(fm_launch_cols(m, A, true, st));
        if (p->update_w0 && nb > 0) FM_TRY(fm_bias_step(m, w0, m->scal + 1, p->eta, nullptr, st));
    }
    if (lazy) {
        ColArgs F;
        col_args(m->B, F);
        FM_TRY(fm_launch_cols_flush(m, F, st));
    }
    if (objective != nullptr) {
        FM_TRY(run_forward(m, p, y, w0, w, V, nullptr, nullptr, nullptr, nullptr, nullptr, 1, true, st));
        FM_TRY(fm_reduce_sum(m, w, m->D, 1, true, m->scal + 2, st));
        FM_TRY(fm_reduce_sum(m, V, m->D * (int64_t)p->K, 1, true, m->scal + 3, st));
        FM_HIP(m, hipMemcpyAsync(m->h_scal, m->scal, 4 * sizeof(double), hipMemcpyDeviceToHost, st));
        FM_HIP(m, hipStreamSynchronize(st));
        objective[0] = (double)p->loss_scale * m->h_scal[0];
        objective[1] = 0.5 * (double)p->lambda_w * m->h_scal[2] + 0.5 * (double)p->lambda_v * m->h_scal[3];
    }
    return FM_OK;
}

extern "C" int fm_get_aux(const fm_matrix* m, float* a, float* G, float* q, float* r, void* hip_stream)
{
    if (m == nullptr) return FM_EINVAL;
    fm_matrix* mm = const_cast<fm_matrix*>(m);
    if (m->wsK == 0 || !m->aux_held) return fm_fail(mm, FM_ESTATE, "no aggregates held");
    if ((a != nullptr || q != nullptr) && !m->aux_full)
        return fm_fail(mm, FM_ESTATE, "a and q are only held after a stratified call");
    hipStream_t st = (hipStream_t)hip_stream;
    FM_TRY(fm_unpack_aux(mm, a, G, q, r, st));
    return FM_OK;
}


// ------------------------------------------------------------- settings ----

extern "C" int fm_set_option(fm_matrix* m, int32_t option, int32_t value)
{
    if (m == nullptr) return FM_EINVAL;
    switch (option) {
        case FM_OPT_AUX_PLANAR:
            if (m->opt.aux_planar != (value != 0)) {
                FM_HIP(m, hipDeviceSynchronize());
                fm_drop_workspace(m);  // the aggregates change layout
                m->opt.aux_planar = value != 0;
            }
            return FM_OK;
        case FM_OPT_SIDE_STREAMS:
            m->opt.side_streams = value != 0;
            fm_drop_graph(m);
            return FM_OK;
        case FM_OPT_LAZY_REG:
            m->opt.lazy_reg = value != 0;
            return FM_OK;
        case FM_OPT_DENSE_ROWS:
            m->opt.dense_rows = value != 0;
            return FM_OK;
        case FM_OPT_GRAPH:
            if (value < 0 || value > 2) return fm_fail(m, FM_EINVAL, "graph mode %d outside 0..2", value);
            m->opt.graph = value;
            return FM_OK;
    }
    return fm_fail(m, FM_EINVAL, "unknown option %d", option);
}

extern "C" int fm_set_tuning(fm_matrix* m, int32_t seg, int32_t panel, int32_t heavy_per_panel, int32_t vlong,
                             int32_t min_panels)
{
    if (m == nullptr) return FM_EINVAL;
    if (m->has_csc) return fm_fail(m, FM_ESTATE, "fm_set_tuning must come before fm_build_csc");
    FmTune& t = m->tune;
    if (seg > 0) t.seg = t.seg_strat = seg < 16 ? 16 : seg;
    if (panel > 0) t.panel = panel < 64 ? 64 : panel;
    if (heavy_per_panel > 0) t.heavy_per_panel = heavy_per_panel;
    if (vlong > 0) t.vlong = vlong;
    if (min_panels > 0) t.min_panels = min_panels;
    return FM_OK;
}

extern "C" int fm_set_tile_tuning(fm_matrix* m, int32_t tile_rows, int32_t min_per_tile, int32_t tile_seg)
{
    if (m == nullptr) return FM_EINVAL;
    if (m->has_csc) return fm_fail(m, FM_ESTATE, "fm_set_tile_tuning must come before fm_build_csc");
    FmTune& t = m->tune;
    if (tile_rows > 0) t.tile = tile_rows < 64 ? 64 : tile_rows;
    if (min_per_tile >= 0) t.tile_min = min_per_tile;
    if (tile_seg > 0) t.tile_seg = tile_seg < 16 ? 16 : tile_seg;
    return FM_OK;
}
