// Internal declarations shared by the translation units of libfm_mi355x.so.
// gfx950 only: 64-lane wavefronts are assumed throughout.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <initializer_list>
#include <string>
#include <vector>

#include "fm.h"

constexpr int FM_WAVE = 64;
constexpr int FM_BLOCK = 256;             // threads per workgroup of the pass kernels
constexpr int FM_WAVES = FM_BLOCK / FM_WAVE;
constexpr int FM_MAXP = 1 << 20;       // row blocks / batches
constexpr int FM_MAXP_CELLS = 4096;     // the P x P table of entries per cell is only kept up to this P
constexpr int FM_XCDS = 8;                // L2 domains; workgroup b runs on XCD b % 8

// Tunables of the column-side work decomposition, per handle (fm_set_tuning, fm_set_tile_tuning;
// tile, tile_min < 0, tile_seg: 0 or negative = chosen per latent size, see fm_tile_shape).
struct FmTune {
    int seg = 256;             // entries per work item of a long column
    int panel = 32768;         // rows per panel of the L2-blocked traversal of heavy columns
    int heavy_per_panel = 16;  // a column is heavy if it averages at least this many entries per panel
    int vlong = 512;           // columns with more items than this are finished by a whole workgroup
    int min_panels = 8 * 8;    // the panel order is used only for matrices with at least this many panels
    int tile = 0;              // rows per LDS tile of the kernel for dense-ish columns
    int tile_min = -1;         // a column is dense-ish if it averages this many entries per tile (0: none)
    int tile_seg = 0;          // entries per item inside a tile
    int seg_strat = 0;         // `seg` of the per-stratum and per-batch matrices (fm_set_tuning sets both); 0: automatic
};

// Per-handle switches between code paths that compute the same thing (fm_set_option).
struct FmOptions {
    bool aux_planar = false;   // planar aggregates for every K (default: packed rows when [G | r] fits one line)
    bool side_streams = true;  // column kernels that touch disjoint columns overlap on internal side streams
    bool lazy_reg = true;      // regulariser-only steps of a stratified or mini-batch epoch are postponed
    int graph = 1;             // stratified epoch from a captured graph: 0 never, 1 when launch-bound, 2 always
    bool dense_rows = true;    // matrices that store every column in every row take the dense (MFMA) kernels
};

// Where the handle keeps the aggregates.  Packed (when [G | r] fits one 128-byte line: K % 4 == 0,
// K <= 28): one row [G_0..G_{K-1}, r, a, q, pad] per example with a stride that is a multiple of
// 16 floats.  Planar otherwise: G dense [N x K], then r, a, q as dense vectors.
struct FmAux {
    float *G, *r, *a, *q;
    int64_t gs, ss;
};
struct fm_matrix;
bool fm_aux_packed(const fm_matrix* m, int32_t K);
// floats per row of partial sums [acc_0..acc_{K-1} | gw | s2 | pad]: a multiple of 32 (128 bytes)
inline int64_t fm_part_stride(int32_t K) { return ((int64_t)K + 2 + 31) / 32 * 32; }
// How the column kernels read the aggregate rows (ColArgs::packed).
enum { FM_PLANAR = 0, FM_PACKED_LANE = 1 };
int fm_cols_packed_mode(const fm_matrix* m, int32_t K);
int64_t fm_aux_floats(const fm_matrix* m, int32_t K);
FmAux fm_aux_layout(const fm_matrix* m, int32_t K);

enum fm_kernel_id {
    FMK_ROWS_FORWARD = 0,
    FMK_ROWS_REFRESH,
    FMK_COLS,
    FMK_COLS_LONG,
    FMK_COLS_TILE,
    FMK_COLS_FINISH,
    FMK_REDUCE,
    FMK_BIAS,
    FMK_COUNT
};

// Work items for columns longer than `seg` entries (of one matrix, or of all strata
// concatenated).  Offsets in item_beg are global offsets into the entry arrays.  Items of
// a column are numbered consecutively (long_first); partial sums live at the item id.
struct LongIndex {
    int64_t nlong = 0, nitems = 0;
    int32_t* long_col = nullptr;    // [nlong] column id
    int64_t* long_first = nullptr;  // [nlong+1] first item of each long column
    int32_t* item_col = nullptr;    // [nitems]
    int64_t* item_beg = nullptr;    // [nitems]
    int32_t* item_len = nullptr;    // [nitems]
    std::vector<int64_t> h_long_off, h_item_off;  // per-stratum ranges (size P+1), or {0,nlong}
    // non-empty columns with at most `seg` entries, in column order (per stratum: h_short_off)
    int64_t nshort = 0;
    int32_t* short_col = nullptr;
    int64_t* short_beg = nullptr;   // per-stratum and per-batch indices only: first entry and number of
    int32_t* short_len = nullptr;   // entries of every listed column (the full matrix has its colptr)
    std::vector<int64_t> h_short_off;
    // processing order of the full matrix: FM_XCDS lists of item ids, list x walked by the
    // workgroups that run on XCD x, heavy columns panel by panel (order == nullptr: id order)
    uint32_t* order = nullptr;      // [nitems]
    int64_t* ord_beg = nullptr;     // [nitems] item_beg / item_len in processing order
    int32_t* ord_len = nullptr;
    int64_t list_off[FM_XCDS + 1] = {0};
    int64_t list_mid[FM_XCDS] = {0};  // in list x, positions from list_mid[x] on are not panel items
    // items of dense-ish columns: positions list_off[FM_XCDS]..nitems of `order`, sorted by row tile
    int64_t tile_rows = 0, ntiles = 0;
    int64_t* tile_ptr = nullptr;    // [ntiles+1] positions in `order`
    int32_t* vlong = nullptr;       // [nvlong] indices into long_col of columns with > vlong items
    int64_t nvlong = 0;
};

struct ProfRec {
    int id;
    hipEvent_t a, b;
};

struct fm_matrix {
    int64_t N = 0, D = 0, nnz = 0;
    FmTune tune;
    FmOptions opt;
    unsigned tile_attr_set = 0;  // bit log2(L): k_cols_tile<L> has been given its dynamic-LDS limit
    // CSR
    int64_t* rowptr = nullptr;
    int32_t* col = nullptr;
    float* val = nullptr;
    // CSC
    bool has_csc = false;
    int64_t* colptr = nullptr;
    int32_t* crow = nullptr;
    float* cval = nullptr;
    LongIndex lfull;
    int lfull_shape[3] = {0, 0, 0};  // tile rows, entries per tile that make a column dense-ish, item length in a tile
    // double partition and per-stratum matrices
    int32_t P = 0;
    std::vector<int64_t> h_rb, h_cb, h_cell_nnz, h_strat_nnz_off;  // bounds, P*P table, P+1 offsets
    int32_t* d_place = nullptr;    // [D] worker every column starts at (fm_partition_placed), nullptr: its column block
    float* d_rho = nullptr;        // [P] share |I_p|/N of the regulariser that a step on row block p applies
    int64_t* d_rb = nullptr;       // [P+1] row block bounds
    int64_t* d_bb = nullptr;       // [B+1] batch bounds
    int32_t* lazy_last = nullptr;  // [D] see ColArgs::lazy_last
    // Per-stratum matrices: the entries of X ordered by (stratum, row, column) in s_col/s_val and by
    // (stratum, column, row) in s_row/s_cval.  No pointer array over all P*N rows or P*D columns: only
    // the rows (columns) that have an entry in a stratum are listed, with the offset of their entries.
    int32_t* s_col = nullptr;
    float* s_val = nullptr;
    int32_t* s_row = nullptr;
    float* s_cval = nullptr;
    LongIndex lstrat;
    int32_t* s_touched = nullptr;  // per stratum: the rows with at least one entry there, ascending
    int64_t* s_touched_beg = nullptr;  // [ntouched+1] where the entries of each listed row begin
    int64_t ntouched = 0;
    std::vector<int64_t> h_touch_off;  // [P+1] offsets into s_touched
    int32_t* s_ncol = nullptr;      // the same for the columns of every stratum
    int64_t* s_ncol_beg = nullptr;  // [nncol+1]
    int64_t nncol = 0;
    std::vector<int64_t> h_ncol_off;  // [P+1]
    int32_t* col_mark = nullptr;    // [D] zero between launches; see ColArgs::mark
    // row batches of the mini-batch epoch: per batch the CSC of the matrix restricted to its rows
    int32_t B = 0;
    std::vector<int64_t> h_bb, h_batch_nnz_off;  // [B+1] row bounds, [B+1] offsets into b_row/b_cval
    int32_t* b_row = nullptr;     // entries ordered by (batch, column, row)
    float* b_cval = nullptr;
    int32_t* b_ncol = nullptr;      // the columns with an entry in every batch, and where their entries begin
    int64_t* b_ncol_beg = nullptr;  // [nbcol+1]
    int64_t nbcol = 0;
    std::vector<int64_t> h_bcol_off;  // [B+1]
    LongIndex lbatch;
    float* d_brho = nullptr;  // [B] share |I_b|/N
    // workspace, sized for wsK
    int32_t wsK = 0;
    float* aux = nullptr;   // aggregates, see fm_aux_layout
    _Float16* Vh = nullptr; // [D*K] half-precision copy of V for passes with half_gather (allocated on first use)
    int32_t VhK = 0;        // the K it was sized for
    // Every row stores all D columns in order (col[e] == e % D): `val` is then a dense row-major N x D
    // matrix and whole-matrix passes can run as dense contractions.  ldense: the partial sums of column j
    // over chunk c of the rows live at item j * dense_chunks + c.
    bool is_dense = false;
    LongIndex ldense;
    int64_t dense_chunk_rows = 0, dense_chunks = 0;
    float* dV = nullptr;    // [D*K] last step's change of V
    float2* dwn = nullptr;  // [D] (change of w_j, change of |v_j|^2)
    float* part = nullptr;      // [max items * part_stride(K)] partial sums of the items, see fm_part_stride
    float* row_part = nullptr;  // [2 * row blocks]: loss, sum r
    double* scal = nullptr;     // device scalars: 0 loss, 1 sum r, 2 |w|^2, 3 |V|^2
    double* h_scal = nullptr;   // pinned mirror
    bool aux_full = false;      // a, q valid (not only G, r)
    bool aux_held = false;      // the aggregate rows hold the result of a pass (fm_get_aux may read them)
    // side streams so that the LDS-bound and the memory-bound column kernels overlap
    hipStream_t side1 = nullptr, side2 = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join1 = nullptr, ev_join2 = nullptr;
    int side_state = 0;  // 0 not tried, 1 ready, -1 unavailable or disabled
    // the stratified epoch as a captured graph (launch-bound for small matrices), replayed while the
    // caller passes the same parameters and arrays; built on an internal stream
    hipStream_t gstream = nullptr;
    hipEvent_t g_in = nullptr, g_out = nullptr;
    hipGraphExec_t gexec = nullptr;
    fm_params gkey_p = {};
    const void* gkey_ptr[4] = {nullptr, nullptr, nullptr, nullptr};
    bool gkey_lazy = false;
    int graph_state = 0;  // 0 not tried, 1 stream and events ready, -1 unavailable
    // profiling
    bool prof = false;
    std::vector<ProfRec> prof_recs;
    std::vector<hipEvent_t> prof_pool;
    int64_t prof_launches[FMK_COUNT] = {0};
    double prof_ms[FMK_COUNT] = {0};
    // bookkeeping
    std::vector<void*> allocs;
    std::string err;
};

// ---- helpers (fm_api.hip) ----
int fm_fail(fm_matrix* m, int code, const char* fmt, ...);
// the kernels read and write the arrays that hold K floats per row four floats at a time
inline int fm_check_vec_aligned(fm_matrix* m, std::initializer_list<const void*> arrays)
{
    for (const void* a : arrays)
        if ((reinterpret_cast<uintptr_t>(a) & 15u) != 0)
            return fm_fail(m, FM_EINVAL, "device arrays with K floats per row (V, G, grad_V) must be 16-byte aligned");
    return FM_OK;
}
int fm_dev_alloc(fm_matrix* m, void** p, size_t bytes);
void fm_dev_free(fm_matrix* m, void* p);
void fm_drop_workspace(fm_matrix* m);  // forces reallocation after the structures changed
void fm_drop_graph(fm_matrix* m);      // a captured epoch holds pointers into the workspace and the structures
bool fm_side_streams(fm_matrix* m);    // creates them on first use; false if switched off or unavailable

#define FM_HIP(m, expr)                                                                  \
    do {                                                                                 \
        hipError_t e__ = (expr);                                                         \
        if (e__ != hipSuccess)                                                           \
            return fm_fail((m), FM_EHIP, "%s failed: %s", #expr, hipGetErrorString(e__)); \
    } while (0)

#define FM_TRY(expr)          \
    do {                      \
        int rc__ = (expr);    \
        if (rc__ != FM_OK) return rc__; \
    } while (0)

struct ProfScope {
    fm_matrix* m;
    hipStream_t st;
    int id;
    hipEvent_t a = nullptr, b = nullptr;
    ProfScope(fm_matrix* m_, hipStream_t st_, int id_);
    ~ProfScope();
};

// ---- build (fm_build.hip) ----
int fm_scan_exclusive_i64(fm_matrix* m, int64_t* d, int64_t n, hipStream_t st);
int fm_sort_by_key_u32(fm_matrix* m, uint32_t* keys, uint32_t* idx, uint32_t* keys_alt, uint32_t* idx_alt,
                       int64_t n, int bits, hipStream_t st, bool* result_in_alt);
// ptr[c], ptr[c+1] bound the entries of list position c = 0..ncols_total-1; ids[c] is its column;
// h_bounds[s] (nstrata+1 values) is the first list position of stratum s
int fm_build_long_index(fm_matrix* m, const int64_t* ptr, const int32_t* ids, int64_t ncols_total,
                        const std::vector<int64_t>& h_bounds, int32_t nstrata, LongIndex* out, hipStream_t st);
// lfull, with the panel order of heavy columns and the LDS tiles shaped for latent size K (0: unknown)
int fm_build_full_index(fm_matrix* m, int32_t K, hipStream_t st);
void fm_tile_shape(const fm_matrix* m, int32_t K, int* tile_rows, int* tile_min, int* tile_seg);
int fm_ensure_lazy(fm_matrix* m);  // allocates lazy_last on first use

// ---- pass kernels (fm_rows.hip / fm_cols.hip / fm_reduce.hip) ----
struct RowArgs {
    int64_t N;
    int32_t K;
    const int64_t* rowptr;
    const int32_t* col;
    const float* val;
    const float* w0;    // device scalar
    const float* w;     // forward: weights
    const float* V;     // forward: factors ; refresh: dV
    const _Float16* Vh; // forward, nullable: gather the rows of V from this half-precision copy instead
    const float2* dwn;  // refresh: (dw_j, dn_j)
    const float* y;     // nullable
    float *yhat, *a, *G, *q, *r;  // forward: nullable outputs ; refresh: in/out aggregates
    int64_t gs;         // floats between consecutive rows of G
    int64_t ss;         // floats between consecutive rows of r, a, q (1, or the aggregate row stride)
    int32_t whole_rows; // forward into packed aggregate rows: write r, a, q and the padding with G
    float* row_part;    // nullable: [2*gridDim] loss and sum r per block
    int32_t dense_D;      // forward: > 0 when `val` is a dense row-major N x dense_D matrix (col is then not read)
    const int32_t* rows;  // nullable: the launch covers rows[0..N) instead of rows 0..N-1, and
                          // rowptr[k], rowptr[k+1] bound the entries of rows[k]
    int32_t loss;
    float s;
};
int fm_launch_rows(fm_matrix* m, const RowArgs& A, bool refresh, hipStream_t st);
int64_t fm_rows_grid(int64_t N, int32_t K);
// once per device, with that device current: resolves the address of the static scratch array of
// fm_forward_noalloc (fm_noalloc.hip); called when a handle is created
int fm_noalloc_init_device(fm_matrix* m);
int fm_pack_aux(fm_matrix* m, const float* r, const float* G, hipStream_t st);  // packed layout only
int fm_to_half(fm_matrix* m, const float* x, _Float16* out, int64_t n, hipStream_t st);  // round to nearest even
// dense matrices (fm_dense.hip)
int fm_dense_detect(fm_matrix* m, hipStream_t st);           // sets is_dense
bool fm_dense_shape_ok(const fm_matrix* m, int32_t K);       // the dense kernels exist for this D and K
int fm_dense_build_index(fm_matrix* m, hipStream_t st);      // ldense, dense_chunk_rows, dense_chunks
int fm_launch_rows_dense(fm_matrix* m, const RowArgs& A, hipStream_t st);
struct ColArgs;
int fm_launch_cols_dense(fm_matrix* m, const ColArgs& A, hipStream_t st);  // partial sums only; the finish kernels follow
int fm_unpack_aux(fm_matrix* m, float* a, float* G, float* q, float* r, hipStream_t st);

struct ColArgs {
    int64_t D;
    int32_t K;
    const int64_t* ptr;  // [D+1] global offsets of the full matrix; nullptr for a stratum or batch (short_beg/len, items)
    const int32_t* row;
    const float* val;
    const float* r;
    const float* G;
    int64_t gs, rs;  // row strides of G and r in floats
    // dense matrices (every row stores all D columns): X = the CSR values as a row-major N x D matrix; wavefront c
    // sums rows [c * chunk_rows, (c+1) * chunk_rows) and stores column j's partial sums at item j * nchunks + c
    const float* X;
    int64_t chunk_rows, nchunks;
    int32_t packed;  // FM_PLANAR, or FM_PACKED_LANE: G rows are packed aggregate rows [G | r | a | q | pad]
    float* w;        // updated in place when update
    float* V;
    float* grad_w;   // !update: outputs (nullable)
    float* grad_V;
    float* dV;       // delta outputs (nullable)
    float2* dwn;
    const int32_t* short_col;  // list of the short non-empty columns of this launch
    const int64_t* short_beg;  // with ptr == nullptr: first entry and number of entries of every listed column
    const int32_t* short_len;
    int64_t nshort;
    // nullable, with ptr == nullptr and steps taken at once: every column that takes its step from data sets
    // mark[j] = 1, and the kernel of the columns without entries skips the marked ones and clears the mark
    int32_t* mark;
    float lambda_w, lambda_v, eta;
    // regulariser share: rho = 1 when rho == nullptr, else rho[p] = |I_p|/N with p = (c(j) - s) mod P, where
    // c(j) = place[j], or the column block of j when place == nullptr
    const int32_t* place;
    const float* rho;
    const int64_t* rb;           // with rho: [P+1] bounds of the row blocks (strata) or batches
    float rho_small, rho_big;    // with rho: the shares of a block of floor(N/P) rows and of one more
    int64_t N;
    int32_t P, s;
    int32_t batch;  // 1: steps are row batches, step t acts on row block t (else on (colblock - t) mod P)
    // nullable, update only: lazy_last[j] = number of strata of this epoch whose step column j has
    // taken.  A column that is empty in a cell only feels the regulariser there; with this array
    // those steps are postponed until the column next has entries (or the epoch ends) and then
    // taken as one multiplication, so no pass over the columns that are empty in a stratum is needed.
    int32_t* lazy_last;
    // long-column items
    const int32_t* long_col;
    const int64_t* long_first;
    const int32_t* item_col;
    const int64_t* item_beg;
    const int32_t* item_len;
    int64_t nlong, nitems;        // counts of this launch
    int64_t long_base, item_base;  // first long column / first item of this launch (absolute ids)
    const uint32_t* order;         // nullable: item ids in processing order, FM_XCDS lists
    const int64_t* ord_beg;        // with order: item_beg / item_len in processing order
    const int32_t* ord_len;
    int64_t list_off[FM_XCDS + 1];
    int64_t list_mid[FM_XCDS];
    int64_t tile_rows, ntiles;     // dense-ish columns: items sorted by row tile, after the lists
    const int64_t* tile_ptr;
    int32_t lin_mode;              // k_cols_long: take positions lin_base.. of `order` in sequence
    int64_t lin_base, lin_count;
    const int32_t* vlong;          // nullable: long columns finished by a whole workgroup
    int64_t nvlong;
    int32_t vlong_items;           // threshold that defines vlong
    float* part;                    // rows [acc | gw | s2 | pad] of ps floats, indexed by absolute item id
    int64_t ps;
};
int fm_launch_cols(fm_matrix* m, const ColArgs& A, bool update, hipStream_t st);
// takes the postponed regulariser steps of every column up to stratum A.s (exclusive)
int fm_launch_cols_flush(fm_matrix* m, const ColArgs& A, hipStream_t st);

constexpr int FM_REDUCE_TMP = 2048;  // doubles of stage-1 scratch a reduction may use
// tmp: FM_REDUCE_TMP doubles of device scratch, or nullptr for the handle's own
int fm_reduce_pairs(fm_matrix* m, const float* part, int64_t nblocks, double* out2, hipStream_t st,
                    double* tmp = nullptr);
int fm_reduce_sum(fm_matrix* m, const float* x, int64_t n, int64_t stride, bool square, double* out1, hipStream_t st);
int fm_reduce_eval(fm_matrix* m, const float* yhat, const float* y, int64_t n, int what, double* out1, hipStream_t st);
int fm_fill_i32(fm_matrix* m, int32_t* x, int64_t n, int32_t v, hipStream_t st);
int fm_bias_step(fm_matrix* m, float* w0, const double* rsum, float eta, float* grad_w0_out, hipStream_t st);

// lanes per row/column group and floats per lane for a given K; false if K unsupported
bool fm_shape_for_K(int32_t K, int* vec, int* lanes);
