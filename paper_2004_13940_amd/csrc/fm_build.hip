// Integer-only builders: exclusive scan, stable LSD radix sort, CSR->CSC transpose,
// the per-stratum matrices of the double partition, and the work-item lists for long
// columns.  Everything here is deterministic (integer atomics are only used for
// counts, whose totals do not depend on the order of the additions).
#include "fm_device.h"
#include "fm_internal.h"

namespace {

// ------------------------------------------------------------------ scan ----
constexpr int SCAN_T = 256;
constexpr int SCAN_E = 8;
constexpr int SCAN_TILE = SCAN_T * SCAN_E;

// exclusive prefix of one int64 per thread across the 256 threads of a block
__device__ __forceinline__ int64_t block_exclusive_256(int64_t v, int64_t (*sh)[SCAN_T], int64_t* total)
{
    const int t = threadIdx.x;
    sh[0][t] = v;
    __syncthreads();
    int cur = 0;
    for (int o = 1; o < SCAN_T; o <<= 1) {
        int64_t x = sh[cur][t];
        if (t >= o) x += sh[cur][t - o];
        sh[cur ^ 1][t] = x;
        __syncthreads();
        cur ^= 1;
    }
    const int64_t incl = sh[cur][t];
    if (total != nullptr) *total = sh[cur][SCAN_T - 1];
    __syncthreads();
    return incl - v;
}

__global__ __launch_bounds__(SCAN_T) void k_scan_sums(const int64_t* __restrict__ d, int64_t n,
                                                      int64_t* __restrict__ sums)
{
    __shared__ int64_t sh[2][SCAN_T];
    const int64_t base = (int64_t)blockIdx.x * SCAN_TILE;
    int64_t v = 0;
    for (int u = 0; u < SCAN_E; ++u) {
        const int64_t i = base + (int64_t)u * SCAN_T + threadIdx.x;
        if (i < n) v += d[i];
    }
    int64_t total;
    block_exclusive_256(v, sh, &total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(SCAN_T) void k_scan_apply(int64_t* __restrict__ d, int64_t n,
                                                       const int64_t* __restrict__ offs)
{
    __shared__ int64_t sh[2][SCAN_T];
    const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_E;
    int64_t x[SCAN_E];
    int64_t tot = 0;
#pragma unroll
    for (int u = 0; u < SCAN_E; ++u) {
        x[u] = (base + u < n) ? d[base + u] : 0;
        tot += x[u];
    }
    int64_t run = block_exclusive_256(tot, sh, nullptr) + (offs != nullptr ? offs[blockIdx.x] : 0);
#pragma unroll
    for (int u = 0; u < SCAN_E; ++u) {
        if (base + u < n) d[base + u] = run;
        run += x[u];
    }
}

// ------------------------------------------------------------ radix sort ----
constexpr int RS_T = 256;
constexpr int RS_ROUNDS = 8;
constexpr int RS_TILE = RS_T * RS_ROUNDS;

__global__ __launch_bounds__(RS_T) void k_radix_hist(const uint32_t* __restrict__ keys, int64_t n, int shift,
                                                     int64_t* __restrict__ hist, int64_t nblocks)
{
    __shared__ unsigned int h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * RS_TILE;
    for (int u = 0; u < RS_ROUNDS; ++u) {
        const int64_t i = base + (int64_t)u * RS_T + threadIdx.x;
        if (i < n) atomicAdd(&h[(keys[i] >> shift) & 255u], 1u);
    }
    __syncthreads();
    hist[(int64_t)threadIdx.x * nblocks + blockIdx.x] = (int64_t)h[threadIdx.x];
}

// Stable scatter: elements of a block are taken in memory order (round by round,
// lane by lane); an element's slot is the scanned start of (digit, block) plus the
// number of same-digit elements before it in the block.
__global__ __launch_bounds__(RS_T) void k_radix_scatter(const uint32_t* __restrict__ keys_in,
                                                        const uint32_t* __restrict__ idx_in,
                                                        uint32_t* __restrict__ keys_out,
                                                        uint32_t* __restrict__ idx_out, int64_t n, int shift,
                                                        const int64_t* __restrict__ hist, int64_t nblocks)
{
    __shared__ int64_t base[256];
    __shared__ unsigned int wcnt[RS_T / 64][256];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    base[tid] = hist[(int64_t)tid * nblocks + blockIdx.x];
    const int64_t tile = (int64_t)blockIdx.x * RS_TILE;
    for (int u = 0; u < RS_ROUNDS; ++u) {
#pragma unroll
        for (int k = 0; k < RS_T / 64; ++k) wcnt[k][tid] = 0;
        __syncthreads();
        const int64_t i = tile + (int64_t)u * RS_T + tid;
        const bool valid = i < n;
        const uint32_t key = valid ? keys_in[i] : 0u;
        const uint32_t dg = (key >> shift) & 255u;
        unsigned long long mask = __ballot(valid);
#pragma unroll
        for (int bit = 0; bit < 8; ++bit) {
            const bool bb = (dg >> bit) & 1u;
            const unsigned long long bal = __ballot(bb);
            mask &= bb ? bal : ~bal;
        }
        const unsigned int rank = __popcll(mask & ((1ull << lane) - 1ull));
        if (valid && rank == 0) wcnt[wave][dg] = (unsigned int)__popcll(mask);
        __syncthreads();
        if (valid) {
            unsigned int off = 0;
            for (int k = 0; k < wave; ++k) off += wcnt[k][dg];
            const int64_t dst = base[dg] + off + rank;
            keys_out[dst] = key;
            idx_out[dst] = idx_in[i];
        }
        __syncthreads();
        unsigned int add = 0;
#pragma unroll
        for (int k = 0; k < RS_T / 64; ++k) add += wcnt[k][tid];
        base[tid] += add;
    }
}

// ------------------------------------------------------------- transpose ----
__global__ void k_init_keys(const int32_t* __restrict__ col, uint32_t* __restrict__ keys,
                            uint32_t* __restrict__ idx, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        keys[i] = (uint32_t)col[i];
        idx[i] = (uint32_t)i;
    }
}

// owner of entry e in a pointer array ptr[0..n]: the k with ptr[k] <= e < ptr[k+1]
__device__ __forceinline__ int64_t owner_of(const int64_t* __restrict__ ptr, int64_t n, int64_t e)
{
    int64_t lo = 0, hi = n;
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (ptr[mid] <= e) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ void k_gather_transposed(const uint32_t* __restrict__ perm, const int64_t* __restrict__ ptr, int64_t nown,
                                    const float* __restrict__ val, int32_t* __restrict__ owner_out,
                                    float* __restrict__ val_out, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        const int64_t e = perm[i];
        owner_out[i] = (int32_t)owner_of(ptr, nown, e);
        val_out[i] = val[e];
    }
}

// ptr[j] = number of sorted keys smaller than j, j = 0..ncols
__global__ void k_ptr_from_sorted(const uint32_t* __restrict__ keys, int64_t n, int64_t ncols,
                                  int64_t* __restrict__ ptr)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j > ncols) return;
    int64_t lo = 0, hi = n;  // first position with key >= j
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)keys[mid] < j) lo = mid + 1; else hi = mid;
    }
    ptr[j] = lo;
}

// -------------------------------------------------------------- partition ----
// Stratum of every stored entry; `major` is the pointer array of the orientation
// being processed (rowptr for CSR, colptr for CSC) and `minor` its index array.
__global__ void k_stratum_keys(const int64_t* __restrict__ major, int64_t nmajor, const int32_t* __restrict__ minor,
                               int64_t n, int64_t N, int64_t D, int32_t P, int by_rows,
                               const int32_t* __restrict__ place, uint32_t* __restrict__ keys, uint32_t* __restrict__ idx)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n) return;
    const int64_t mj = owner_of(major, nmajor, e);
    const int64_t mn = minor[e];
    const int64_t i = by_rows == 1 ? mj : mn;
    const int64_t j = by_rows == 1 ? mn : mj;
    const int32_t p = fm_block_of(i, N, P);
    int32_t s;
    if (by_rows == 2) {  // row batches: the key is the row block alone
        s = p;
    } else {
        const int32_t q = place != nullptr ? place[j] : fm_block_of(j, D, P);
        s = (q - p) % P;
        if (s < 0) s += P;
    }
    keys[e] = (uint32_t)s;
    idx[e] = (uint32_t)e;
}

// major index (row of a CSR entry, column of a CSC entry) of every entry of a permuted order
__global__ void k_major_of(const uint32_t* __restrict__ perm, const int64_t* __restrict__ major, int64_t nmajor,
                           int32_t* __restrict__ out, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = (int32_t)owner_of(major, nmajor, perm[i]);
}

// flag[i] = 1 where entry i (in stratum order) opens a new (stratum, major) pair
__global__ void k_head_flags(const uint32_t* __restrict__ keys, const int32_t* __restrict__ maj, int64_t n,
                             int64_t* __restrict__ flag)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) flag[i] = (i == 0 || keys[i] != keys[i - 1] || maj[i] != maj[i - 1]) ? 1 : 0;
}

// pos = exclusive scan of the flags: the pairs in order, with their major index and first entry
__global__ void k_compact_heads(const uint32_t* __restrict__ keys, const int32_t* __restrict__ maj,
                                const int64_t* __restrict__ pos, int64_t n, int32_t* __restrict__ nz_major,
                                int64_t* __restrict__ nz_beg)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    if (i == 0 || keys[i] != keys[i - 1] || maj[i] != maj[i - 1]) {
        nz_major[pos[i]] = maj[i];
        nz_beg[pos[i]] = i;
    }
}

// out[t] = number of elements of the ascending array a[0..n) that are smaller than bound[t]
__global__ void k_lower_bounds(const int64_t* __restrict__ a, int64_t n, const int64_t* __restrict__ bound, int64_t nb,
                               int64_t* __restrict__ out)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= nb) return;
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (a[mid] < bound[t]) lo = mid + 1; else hi = mid;
    }
    out[t] = lo;
}

__global__ void k_gather_i64(const int64_t* __restrict__ src, const int64_t* __restrict__ idx, int64_t n,
                             int64_t* __restrict__ out)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) out[t] = src[idx[t]];
}

__global__ void k_gather_pairs(const uint32_t* __restrict__ perm, const int32_t* __restrict__ ind,
                               const float* __restrict__ val, int32_t* __restrict__ ind_out,
                               float* __restrict__ val_out, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        const int64_t e = perm ? (int64_t)perm[i] : i;
        ind_out[i] = ind[e];
        val_out[i] = val[e];
    }
}

// cell[p*P + c] += 1 for every stored entry in row block p whose column belongs to column block c (or was
// placed at worker c); integer atomics: the totals do not depend on the order
__global__ void k_cell_count(const int64_t* __restrict__ rowptr, int64_t N, const int32_t* __restrict__ col, int64_t n,
                             int64_t D, const int32_t* __restrict__ place, int32_t P,
                             unsigned long long* __restrict__ cell)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n) return;
    const int32_t p = fm_block_of(owner_of(rowptr, N, e), N, P);
    const int32_t c = place != nullptr ? place[col[e]] : fm_block_of(col[e], D, P);
    atomicAdd(&cell[(int64_t)p * P + c], 1ull);
}

// ------------------------------------------------------------ long index ----
constexpr int LI_T = 256;
constexpr int LI_E = 4;
constexpr int LI_TILE = LI_T * LI_E;

__global__ __launch_bounds__(LI_T) void k_long_count(const int64_t* __restrict__ ptr, int64_t ncols, int seg,
                                                     int64_t* __restrict__ tile_long, int64_t* __restrict__ tile_items)
{
    __shared__ int64_t sh[2][SCAN_T];
    const int64_t base = (int64_t)blockIdx.x * LI_TILE + (int64_t)threadIdx.x * LI_E;
    int64_t nl = 0, ni = 0;
    for (int u = 0; u < LI_E; ++u) {
        const int64_t c = base + u;
        if (c < ncols) {
            const int64_t len = ptr[c + 1] - ptr[c];
            if (len > seg) {
                nl += 1;
                ni += (len + seg - 1) / seg;
            }
        }
    }
    int64_t t0, t1;
    block_exclusive_256(nl, sh, &t0);
    block_exclusive_256(ni, sh, &t1);
    if (threadIdx.x == 0) {
        tile_long[blockIdx.x] = t0;
        tile_items[blockIdx.x] = t1;
    }
}

__global__ __launch_bounds__(LI_T) void k_long_fill(const int64_t* __restrict__ ptr, int64_t ncols,
                                                    const int32_t* __restrict__ ids, int seg, int with_items,
                                                    const int64_t* __restrict__ tile_long,
                                                    const int64_t* __restrict__ tile_items,
                                                    int32_t* __restrict__ long_col, int64_t* __restrict__ long_vcol,
                                                    int64_t* __restrict__ long_first, int32_t* __restrict__ item_col,
                                                    int64_t* __restrict__ item_beg, int32_t* __restrict__ item_len)
{
    __shared__ int64_t sh[2][SCAN_T];
    const int64_t base = (int64_t)blockIdx.x * LI_TILE + (int64_t)threadIdx.x * LI_E;
    int64_t nl = 0, ni = 0;
    for (int u = 0; u < LI_E; ++u) {
        const int64_t c = base + u;
        if (c < ncols) {
            const int64_t len = ptr[c + 1] - ptr[c];
            if (len > seg) {
                nl += 1;
                ni += (len + seg - 1) / seg;
            }
        }
    }
    int64_t lpos = block_exclusive_256(nl, sh, nullptr) + tile_long[blockIdx.x];
    int64_t ipos = block_exclusive_256(ni, sh, nullptr) + tile_items[blockIdx.x];
    for (int u = 0; u < LI_E; ++u) {
        const int64_t c = base + u;
        if (c >= ncols) break;
        const int64_t b = ptr[c], len = ptr[c + 1] - b;
        if (len <= seg) continue;
        const int32_t j = ids != nullptr ? ids[c] : (int32_t)c;
        long_col[lpos] = j;
        long_vcol[lpos] = c;
        ++lpos;
        if (!with_items) continue;
        long_first[lpos - 1] = ipos;
        for (int64_t o = 0; o < len; o += seg) {
            item_col[ipos] = j;
            item_beg[ipos] = b + o;
            item_len[ipos] = (int32_t)((len - o) < seg ? (len - o) : seg);
            ++ipos;
        }
    }
}


// -------------------------------------------- short non-empty columns ----
// Columns with 1..seg entries, in (virtual) column order: k_cols works through this list;
// empty columns only feel the regulariser and are handled by an elementwise kernel.
__global__ __launch_bounds__(LI_T) void k_short_list(const int64_t* __restrict__ ptr, int64_t ncols,
                                                     const int32_t* __restrict__ ids, int seg,
                                                     int pass, int64_t* __restrict__ tile_cnt,
                                                     int32_t* __restrict__ short_col, int64_t* __restrict__ short_vcol,
                                                     int64_t* __restrict__ short_beg, int32_t* __restrict__ short_len)
{
    __shared__ int64_t sh[2][SCAN_T];
    const int64_t base = (int64_t)blockIdx.x * LI_TILE + (int64_t)threadIdx.x * LI_E;
    int64_t ns = 0;
    for (int u = 0; u < LI_E; ++u) {
        const int64_t c = base + u;
        if (c < ncols) {
            const int64_t len = ptr[c + 1] - ptr[c];
            if (len > 0 && len <= seg) ns += 1;
        }
    }
    int64_t total;
    int64_t pos = block_exclusive_256(ns, sh, &total);
    if (!pass) {
        if (threadIdx.x == 0) tile_cnt[blockIdx.x] = total;
        return;
    }
    pos += tile_cnt[blockIdx.x];
    for (int u = 0; u < LI_E; ++u) {
        const int64_t c = base + u;
        if (c >= ncols) break;
        const int64_t len = ptr[c + 1] - ptr[c];
        if (len > 0 && len <= seg) {
            short_col[pos] = ids != nullptr ? ids[c] : (int32_t)c;
            short_vcol[pos] = c;
            if (short_beg != nullptr) short_beg[pos] = ptr[c];
            if (short_len != nullptr) short_len[pos] = (int32_t)len;
            ++pos;
        }
    }
}

// off[s] = number of list entries whose position in the column list is < bounds[s], s = 0..nstrata
__global__ void k_stratum_offsets(const int64_t* __restrict__ vcol, int64_t n, const int64_t* __restrict__ bounds,
                                  int32_t nstrata, int64_t* __restrict__ off)
{
    const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s > nstrata) return;
    const int64_t bound = bounds[s];
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (vcol[mid] < bound) lo = mid + 1; else hi = mid;
    }
    off[s] = lo;
}


// ---------------------------------------------------- full-matrix items ----
// first position in rows[beg,end) (ascending) whose row is >= bound
__device__ __forceinline__ int64_t first_row_at_least(const int32_t* __restrict__ rows, int64_t beg, int64_t end,
                                                      int64_t bound)
{
    int64_t lo = beg, hi = end;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)rows[mid] < bound) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// Items of every long column of the full matrix.  A column with fewer than heavy_min
// entries is cut into consecutive segments of `seg` entries.  A heavy column is first
// cut at the boundaries of the row panels [b*panel, (b+1)*panel) and every piece then
// into segments of `seg`; its items carry the key (b % FM_XCDS, b / FM_XCDS) so that the
// stable sort by key hands panel b to XCD b % FM_XCDS in ascending panel order.  Other
// items get the last position of the list (slot % FM_XCDS) and run after the panels.
// A column with at least tile_min entries ("dense-ish") is instead cut at the boundaries of
// row tiles of `tile` rows and into segments of `tseg`; its items get the key
// FM_XCDS*(maxpos+1) + tile id, i.e. they sort behind the eight lists, tile by tile, and are
// processed by the kernel that stages a tile of aggregate rows in LDS.
// One workgroup per long column; pass 0 counts, pass 1 fills.
__global__ __launch_bounds__(256) void k_full_items(const int64_t* __restrict__ colptr, const int32_t* __restrict__ crow,
                                                    const int32_t* __restrict__ long_col, int64_t N, int seg,
                                                    int64_t panel, int64_t heavy_min, int64_t maxpos, int64_t tile,
                                                    int64_t tile_min, int tseg, int pass,
                                                    int64_t* __restrict__ nitems, const int64_t* __restrict__ long_first,
                                                    int32_t* __restrict__ item_col, int64_t* __restrict__ item_beg,
                                                    int32_t* __restrict__ item_len, uint32_t* __restrict__ item_key)
{
    __shared__ int64_t sh[2][SCAN_T];
    const int64_t lc = blockIdx.x;
    const int32_t j = long_col[lc];
    const int64_t beg = colptr[j], end = colptr[j + 1], cnt = end - beg;
    const int64_t first = pass ? long_first[lc] : 0;
    const bool tiled = cnt >= tile_min;
    if (!tiled && cnt < heavy_min) {
        const int64_t nit = (cnt + seg - 1) / seg;
        if (!pass) {
            if (threadIdx.x == 0) nitems[lc] = nit;
            return;
        }
        for (int64_t k = threadIdx.x; k < nit; k += blockDim.x) {
            const int64_t slot = first + k;
            item_col[slot] = j;
            item_beg[slot] = beg + k * seg;
            item_len[slot] = (int32_t)((cnt - k * seg) < seg ? (cnt - k * seg) : seg);
            item_key[slot] = (uint32_t)((slot % FM_XCDS) * (maxpos + 1) + maxpos);
        }
        return;
    }
    const int64_t piece = tiled ? tile : panel;  // rows per piece
    const int64_t sg = tiled ? tseg : seg;       // entries per item inside a piece
    const int64_t npieces = (N + piece - 1) / piece;
    int64_t running = 0;
    for (int64_t b0 = 0; b0 < npieces; b0 += blockDim.x) {
        const int64_t b = b0 + threadIdx.x;
        int64_t lo = 0, hi = 0;
        if (b < npieces) {
            lo = first_row_at_least(crow, beg, end, b * piece);
            hi = first_row_at_least(crow, lo, end, (b + 1) * piece);
        }
        const int64_t nb = (hi - lo + sg - 1) / sg;
        int64_t total;
        const int64_t off = block_exclusive_256(nb, sh, &total);
        if (pass) {
            const uint32_t key = tiled ? (uint32_t)(FM_XCDS * (maxpos + 1) + b)
                                       : (uint32_t)((b % FM_XCDS) * (maxpos + 1) + b / FM_XCDS);
            for (int64_t k = 0; k < nb; ++k) {
                const int64_t slot = first + running + off + k;
                item_col[slot] = j;
                item_beg[slot] = lo + k * sg;
                item_len[slot] = (int32_t)((hi - lo - k * sg) < sg ? (hi - lo - k * sg) : sg);
                item_key[slot] = key;
            }
        }
        running += total;
    }
    if (!pass && threadIdx.x == 0) nitems[lc] = running;
}

// tile_ptr[t] = number of sorted keys smaller than base + t, t = 0..ntiles
__global__ void k_tile_ptr(const uint32_t* __restrict__ keys, int64_t n, int64_t base, int64_t ntiles,
                           int64_t* __restrict__ tile_ptr)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t > ntiles) return;
    const int64_t bound = base + t;
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)keys[mid] < bound) lo = mid + 1; else hi = mid;
    }
    tile_ptr[t] = lo;
}

// item records copied into processing order, so that the column kernel streams them
__global__ void k_order_items(const uint32_t* __restrict__ order, int64_t n, const int64_t* __restrict__ item_beg,
                              const int32_t* __restrict__ item_len, int64_t* __restrict__ ord_beg,
                              int32_t* __restrict__ ord_len)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        const uint32_t it = order[i];
        ord_beg[i] = item_beg[it];
        ord_len[i] = item_len[it];
    }
}

__global__ void k_iota_u32(uint32_t* __restrict__ x, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) x[i] = (uint32_t)i;
}

// list_off[x] = number of sorted keys smaller than x * (maxpos+1), x = 0..FM_XCDS
// and list_off[FM_XCDS+1+x] = number of keys smaller than x*(maxpos+1)+maxpos (first non-panel item)
__global__ void k_list_offsets(const uint32_t* __restrict__ keys, int64_t n, int64_t maxpos,
                               int64_t* __restrict__ list_off)
{
    const int x = threadIdx.x;
    if (x > 2 * FM_XCDS) return;
    const int64_t bound = x <= FM_XCDS ? (int64_t)x * (maxpos + 1)
                                       : (int64_t)(x - FM_XCDS - 1) * (maxpos + 1) + maxpos;
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)keys[mid] < bound) lo = mid + 1; else hi = mid;
    }
    list_off[x] = lo;
}

inline unsigned blocks_for(int64_t n, int t) { return (unsigned)((n + t - 1) / t); }

}  // namespace

// ---------------------------------------------------------------- hosts ----

static int bits_for(int64_t maxval)
{
    int b = 0;
    while (b < 32 && ((int64_t)1 << b) <= maxval) ++b;
    return b;
}

int fm_scan_exclusive_i64(fm_matrix* m, int64_t* d, int64_t n, hipStream_t st)
{
    if (n <= 0) return FM_OK;
    const int64_t ntiles = (n + SCAN_TILE - 1) / SCAN_TILE;
    if (ntiles == 1) {
        hipLaunchKernelGGL(k_scan_apply, dim3(1), dim3(SCAN_T), 0, st, d, n, (const int64_t*)nullptr);
        FM_HIP(m, hipGetLastError());
        return FM_OK;
    }
    int64_t* sums = nullptr;
    FM_TRY(fm_dev_alloc(m, (void**)&sums, (size_t)ntiles * sizeof(int64_t)));
    hipLaunchKernelGGL(k_scan_sums, dim3((unsigned)ntiles), dim3(SCAN_T), 0, st, (const int64_t*)d, n, sums);
    FM_HIP(m, hipGetLastError());
    int rc = fm_scan_exclusive_i64(m, sums, ntiles, st);
    if (rc == FM_OK) {
        hipLaunchKernelGGL(k_scan_apply, dim3((unsigned)ntiles), dim3(SCAN_T), 0, st, d, n, (const int64_t*)sums);
        if (hipGetLastError() != hipSuccess) rc = fm_fail(m, FM_EHIP, "scan apply launch failed");
    }
    if (hipStreamSynchronize(st) != hipSuccess && rc == FM_OK) rc = fm_fail(m, FM_EHIP, "scan failed");
    fm_dev_free(m, sums);
    return rc;
}

int fm_sort_by_key_u32(fm_matrix* m, uint32_t* keys, uint32_t* idx, uint32_t* keys_alt, uint32_t* idx_alt,
                       int64_t n, int bits, hipStream_t st, bool* result_in_alt)
{
    *result_in_alt = false;
    if (n <= 0 || bits <= 0) return FM_OK;
    const int64_t nblocks = (n + RS_TILE - 1) / RS_TILE;
    int64_t* hist = nullptr;
    FM_TRY(fm_dev_alloc(m, (void**)&hist, (size_t)(256 * nblocks) * sizeof(int64_t)));
    int rc = FM_OK;
    uint32_t *ki = keys, *ii = idx, *ko = keys_alt, *io = idx_alt;
    for (int shift = 0; shift < bits && rc == FM_OK; shift += 8) {
        hipLaunchKernelGGL(k_radix_hist, dim3((unsigned)nblocks), dim3(RS_T), 0, st, (const uint32_t*)ki, n, shift,
                           hist, nblocks);
        if (hipGetLastError() != hipSuccess) { rc = fm_fail(m, FM_EHIP, "radix hist launch failed"); break; }
        rc = fm_scan_exclusive_i64(m, hist, 256 * nblocks, st);
        if (rc != FM_OK) break;
        hipLaunchKernelGGL(k_radix_scatter, dim3((unsigned)nblocks), dim3(RS_T), 0, st, (const uint32_t*)ki,
                           (const uint32_t*)ii, ko, io, n, shift, (const int64_t*)hist, nblocks);
        if (hipGetLastError() != hipSuccess) { rc = fm_fail(m, FM_EHIP, "radix scatter launch failed"); break; }
        uint32_t* t = ki; ki = ko; ko = t;
        t = ii; ii = io; io = t;
        *result_in_alt = !*result_in_alt;
    }
    if (hipStreamSynchronize(st) != hipSuccess && rc == FM_OK) rc = fm_fail(m, FM_EHIP, "radix sort failed");
    fm_dev_free(m, hist);
    return rc;
}


// List of the non-empty columns with at most `seg` entries.  ptr[c], ptr[c+1] bound the entries of list
// position c, ids[c] is its column (nullptr: c itself); per stratum when nstrata > 1: h_bounds[s] is the
// first position of stratum s and h_short_off[s] where it starts in the short list.  with_extent: also
// the first entry and the length of every listed column (needed when ptr is not indexed by column).
static int build_short_list(fm_matrix* m, const int64_t* ptr, const int32_t* ids, int64_t ncols_total,
                            const std::vector<int64_t>& h_bounds, int32_t nstrata, int seg, bool with_extent,
                            LongIndex* out, hipStream_t st)
{
    out->nshort = 0;
    out->h_short_off.assign(nstrata + 1, 0);
    if (ncols_total <= 0) return FM_OK;
    const int64_t ntiles = (ncols_total + LI_TILE - 1) / LI_TILE;
    int64_t* tc = nullptr;
    FM_TRY(fm_dev_alloc(m, (void**)&tc, (size_t)(ntiles + 1) * sizeof(int64_t)));
    FM_HIP(m, hipMemsetAsync(tc, 0, (size_t)(ntiles + 1) * sizeof(int64_t), st));
    hipLaunchKernelGGL(k_short_list, dim3((unsigned)ntiles), dim3(LI_T), 0, st, ptr, ncols_total, ids, seg, 0, tc,
                       (int32_t*)nullptr, (int64_t*)nullptr, (int64_t*)nullptr, (int32_t*)nullptr);
    FM_HIP(m, hipGetLastError());
    FM_TRY(fm_scan_exclusive_i64(m, tc, ntiles + 1, st));
    int64_t n = 0;
    FM_HIP(m, hipMemcpyAsync(&n, tc + ntiles, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    FM_HIP(m, hipStreamSynchronize(st));
    if (n > 0) {
        int64_t *vcol = nullptr, *d_off = nullptr, *d_bounds = nullptr;
        FM_TRY(fm_dev_alloc(m, (void**)&out->short_col, (size_t)n * sizeof(int32_t)));
        if (with_extent) {
            FM_TRY(fm_dev_alloc(m, (void**)&out->short_beg, (size_t)n * sizeof(int64_t)));
            FM_TRY(fm_dev_alloc(m, (void**)&out->short_len, (size_t)n * sizeof(int32_t)));
        }
        FM_TRY(fm_dev_alloc(m, (void**)&vcol, (size_t)n * sizeof(int64_t)));
        FM_TRY(fm_dev_alloc(m, (void**)&d_off, (size_t)(nstrata + 1) * sizeof(int64_t)));
        FM_TRY(fm_dev_alloc(m, (void**)&d_bounds, (size_t)(nstrata + 1) * sizeof(int64_t)));
        FM_HIP(m, hipMemcpyAsync(d_bounds, h_bounds.data(), (size_t)(nstrata + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
        hipLaunchKernelGGL(k_short_list, dim3((unsigned)ntiles), dim3(LI_T), 0, st, ptr, ncols_total, ids, seg, 1, tc,
                           out->short_col, vcol, out->short_beg, out->short_len);
        FM_HIP(m, hipGetLastError());
        hipLaunchKernelGGL(k_stratum_offsets, dim3(blocks_for(nstrata + 1, 256)), dim3(256), 0, st, (const int64_t*)vcol,
                           n, (const int64_t*)d_bounds, nstrata, d_off);
        FM_HIP(m, hipGetLastError());
        FM_HIP(m, hipMemcpyAsync(out->h_short_off.data(), d_off, (size_t)(nstrata + 1) * sizeof(int64_t),
                                 hipMemcpyDeviceToHost, st));
        FM_HIP(m, hipStreamSynchronize(st));
        fm_dev_free(m, vcol);
        fm_dev_free(m, d_off);
        fm_dev_free(m, d_bounds);
    }
    out->nshort = n;
    fm_dev_free(m, tc);
    return FM_OK;
}

int fm_build_long_index(fm_matrix* m, const int64_t* ptr, const int32_t* ids, int64_t ncols_total,
                        const std::vector<int64_t>& h_bounds, int32_t nstrata, LongIndex* out, hipStream_t st)
{
    out->nshort = 0;
    out->h_short_off.assign(nstrata + 1, 0);
    out->nlong = out->nitems = 0;
    out->h_long_off.assign(nstrata + 1, 0);
    out->h_item_off.assign(nstrata + 1, 0);
    if (ncols_total <= 0) return FM_OK;
    const int64_t ntiles = (ncols_total + LI_TILE - 1) / LI_TILE;
    int64_t *tl = nullptr, *ti = nullptr;
    FM_TRY(fm_dev_alloc(m, (void**)&tl, (size_t)(ntiles + 1) * sizeof(int64_t)));
    FM_TRY(fm_dev_alloc(m, (void**)&ti, (size_t)(ntiles + 1) * sizeof(int64_t)));
    // Item length.  The launches of one stratum are small: when full-length items would leave a
    // stratum with too few of them to fill the chip, they are halved (more groups to spread over,
    // at the price of more partial sums); fm_set_tuning overrides this.
    int seg = m->tune.seg_strat;
    if (seg <= 0) {
        seg = m->tune.seg;
        FM_HIP(m, hipMemsetAsync(ti, 0, (size_t)(ntiles + 1) * sizeof(int64_t), st));
        FM_HIP(m, hipMemsetAsync(tl, 0, (size_t)(ntiles + 1) * sizeof(int64_t), st));
        hipLaunchKernelGGL(k_long_count, dim3((unsigned)ntiles), dim3(LI_T), 0, st, ptr, ncols_total, seg, tl, ti);
        FM_HIP(m, hipGetLastError());
        FM_TRY(fm_scan_exclusive_i64(m, ti, ntiles + 1, st));
        int64_t n_full = 0;
        FM_HIP(m, hipMemcpyAsync(&n_full, ti + ntiles, sizeof(int64_t), hipMemcpyDeviceToHost, st));
        FM_HIP(m, hipStreamSynchronize(st));
        if (n_full / nstrata < 12288 && seg > 128) seg = 128;
    }
    FM_TRY(build_short_list(m, ptr, ids, ncols_total, h_bounds, nstrata, seg, true, out, st));
    FM_HIP(m, hipMemsetAsync(tl, 0, (size_t)(ntiles + 1) * sizeof(int64_t), st));
    FM_HIP(m, hipMemsetAsync(ti, 0, (size_t)(ntiles + 1) * sizeof(int64_t), st));
    hipLaunchKernelGGL(k_long_count, dim3((unsigned)ntiles), dim3(LI_T), 0, st, ptr, ncols_total, seg, tl, ti);
    FM_HIP(m, hipGetLastError());
    FM_TRY(fm_scan_exclusive_i64(m, tl, ntiles + 1, st));
    FM_TRY(fm_scan_exclusive_i64(m, ti, ntiles + 1, st));
    int64_t nlong = 0, nitems = 0;
    FM_HIP(m, hipMemcpyAsync(&nlong, tl + ntiles, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    FM_HIP(m, hipMemcpyAsync(&nitems, ti + ntiles, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    FM_HIP(m, hipStreamSynchronize(st));
    out->nlong = nlong;
    out->nitems = nitems;
    if (nlong > 0) {
        int64_t* vcol = nullptr;
        FM_TRY(fm_dev_alloc(m, (void**)&out->long_col, (size_t)nlong * sizeof(int32_t)));
        FM_TRY(fm_dev_alloc(m, (void**)&out->long_first, (size_t)(nlong + 1) * sizeof(int64_t)));
        FM_TRY(fm_dev_alloc(m, (void**)&out->item_col, (size_t)nitems * sizeof(int32_t)));
        FM_TRY(fm_dev_alloc(m, (void**)&out->item_beg, (size_t)nitems * sizeof(int64_t)));
        FM_TRY(fm_dev_alloc(m, (void**)&out->item_len, (size_t)nitems * sizeof(int32_t)));
        FM_TRY(fm_dev_alloc(m, (void**)&vcol, (size_t)nlong * sizeof(int64_t)));
        hipLaunchKernelGGL(k_long_fill, dim3((unsigned)ntiles), dim3(LI_T), 0, st, ptr, ncols_total, ids, seg, 1,
                           (const int64_t*)tl, (const int64_t*)ti, out->long_col, vcol, out->long_first,
                           out->item_col, out->item_beg, out->item_len);
        FM_HIP(m, hipGetLastError());
        FM_HIP(m, hipMemcpyAsync(out->long_first + nlong, &nitems, sizeof(int64_t), hipMemcpyHostToDevice, st));
        std::vector<int64_t> h_vcol((size_t)nlong), h_first((size_t)nlong + 1);
        FM_HIP(m, hipMemcpyAsync(h_vcol.data(), vcol, (size_t)nlong * sizeof(int64_t), hipMemcpyDeviceToHost, st));
        FM_HIP(m, hipStreamSynchronize(st));
        FM_HIP(m, hipMemcpy(h_first.data(), out->long_first, (size_t)(nlong + 1) * sizeof(int64_t),
                            hipMemcpyDeviceToHost));
        // per-stratum ranges of the concatenated lists
        int64_t k = 0;
        for (int32_t s = 0; s <= nstrata; ++s) {
            while (k < nlong && h_vcol[(size_t)k] < h_bounds[(size_t)s]) ++k;
            out->h_long_off[s] = k;
            out->h_item_off[s] = h_first[(size_t)k];
        }
        fm_dev_free(m, vcol);
    }
    fm_dev_free(m, tl);
    fm_dev_free(m, ti);
    return FM_OK;
}

// Frees the device arrays of an index and resets it.
static void free_long_index(fm_matrix* m, LongIndex* li)
{
    for (void* p : {(void*)li->long_col, (void*)li->long_first, (void*)li->item_col, (void*)li->item_beg,
                    (void*)li->item_len, (void*)li->short_col, (void*)li->short_beg, (void*)li->short_len, (void*)li->order, (void*)li->ord_beg,
                    (void*)li->ord_len, (void*)li->tile_ptr, (void*)li->vlong})
        if (p != nullptr) fm_dev_free(m, p);
    *li = LongIndex();
}

// Shape of the LDS tiles for N rows and latent size K (K = 0: not known yet).  Explicit settings win;
// else two tiles must fit the LDS of a compute unit (1024 rows only while [G | r] of a row is at most
// 17 floats) and the tile shrinks with the matrix.  Larger tiles mean fewer items, hence fewer partial sums to write and read back.
void fm_tile_shape(const fm_matrix* m, int32_t K, int* tile_rows, int* tile_min, int* tile_seg)
{
    const FmTune& T = m->tune;
    const int64_t N = m->N;
    // one workgroup works on one tile: tall matrices take big tiles (fewer items, hence fewer partial
    // sums), short ones small tiles (enough workgroups to fill the chip)
    int rows = 512, dense = 8, seg = 256;
    if (K > 0 && K % 4 == 0 && K <= 16 && N >= (int64_t(1) << 21)) {
        rows = 1024, dense = 12, seg = 512;
    } else if (N < (int64_t(1) << 17)) {
        rows = 128, dense = 2, seg = 128;
    } else if (N < (int64_t(1) << 18)) {
        rows = 256, dense = 4, seg = 256;
    }
    *tile_rows = T.tile > 0 ? (T.tile < 64 ? 64 : T.tile) : rows;
    *tile_min = T.tile_min >= 0 ? T.tile_min : dense;
    *tile_seg = T.tile_seg > 0 ? T.tile_seg : seg;
}

int fm_build_full_index(fm_matrix* m, int32_t K, hipStream_t st)
{
    LongIndex* out = &m->lfull;
    free_long_index(m, out);
    FmTune T = m->tune;
    fm_tile_shape(m, K, &T.tile, &T.tile_min, &T.tile_seg);
    m->lfull_shape[0] = T.tile;
    m->lfull_shape[1] = T.tile_min;
    m->lfull_shape[2] = T.tile_seg;
    FM_TRY(build_short_list(m, m->colptr, nullptr, m->D, {0, m->D}, 1, m->tune.seg, false, out, st));
    out->nlong = out->nitems = 0;
    out->h_long_off.assign(2, 0);
    out->h_item_off.assign(2, 0);
    const int64_t D = m->D;
    if (D <= 0 || m->nnz == 0) return FM_OK;
    // 1. the long columns, in column order
    const int64_t ntiles = (D + LI_TILE - 1) / LI_TILE;
    int64_t *tl = nullptr, *ti = nullptr, *vcol = nullptr;
    FM_TRY(fm_dev_alloc(m, (void**)&tl, (size_t)(ntiles + 1) * sizeof(int64_t)));
    FM_TRY(fm_dev_alloc(m, (void**)&ti, (size_t)(ntiles + 1) * sizeof(int64_t)));
    FM_HIP(m, hipMemsetAsync(tl, 0, (size_t)(ntiles + 1) * sizeof(int64_t), st));
    FM_HIP(m, hipMemsetAsync(ti, 0, (size_t)(ntiles + 1) * sizeof(int64_t), st));
    hipLaunchKernelGGL(k_long_count, dim3((unsigned)ntiles), dim3(LI_T), 0, st, (const int64_t*)m->colptr, D, T.seg, tl, ti);
    FM_HIP(m, hipGetLastError());
    FM_TRY(fm_scan_exclusive_i64(m, tl, ntiles + 1, st));
    int64_t nlong = 0;
    FM_HIP(m, hipMemcpyAsync(&nlong, tl + ntiles, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    FM_HIP(m, hipStreamSynchronize(st));
    if (nlong == 0) {
        fm_dev_free(m, tl);
        fm_dev_free(m, ti);
        return FM_OK;
    }
    if (nlong > 0x7fffffffLL) return fm_fail(m, FM_ERANGE, "too many long columns");
    FM_TRY(fm_dev_alloc(m, (void**)&out->long_col, (size_t)nlong * sizeof(int32_t)));
    FM_TRY(fm_dev_alloc(m, (void**)&out->long_first, (size_t)(nlong + 1) * sizeof(int64_t)));
    FM_TRY(fm_dev_alloc(m, (void**)&vcol, (size_t)nlong * sizeof(int64_t)));
    hipLaunchKernelGGL(k_long_fill, dim3((unsigned)ntiles), dim3(LI_T), 0, st, (const int64_t*)m->colptr, D,
                       (const int32_t*)nullptr, T.seg, 0,
                       (const int64_t*)tl, (const int64_t*)ti, out->long_col, vcol, (int64_t*)nullptr,
                       (int32_t*)nullptr, (int64_t*)nullptr, (int32_t*)nullptr);
    FM_HIP(m, hipGetLastError());
    // 2. items per long column, then their first ids
    // Panels shrink (down to 1024 rows) so that a matrix of moderate height still has
    // min_panels of them to spread over the XCD lists; the density that makes a column
    // heavy (heavy_per_panel / panel) is kept.
    int64_t panel = T.panel;
    while (panel > 1024 && (m->N + panel - 1) / panel < T.min_panels) panel /= 2;
    const int64_t npanels = (m->N + panel - 1) / panel;
    const double heavy_density = (double)T.heavy_per_panel / (double)T.panel;
    // the panel order pays off only when there are many more panels than XCDs
    const int64_t heavy_min = npanels >= T.min_panels
                                  ? std::max<int64_t>((int64_t)(heavy_density * (double)m->N) + 1, (int64_t)T.seg + 1)
                                  : INT64_MAX;
    const int64_t maxpos = (npanels + FM_XCDS - 1) / FM_XCDS;
    // dense-ish columns (at least tile_min entries per row tile on average) go to the LDS-staged kernel
    const int64_t tile = T.tile;
    const int64_t nrtiles = (m->N + tile - 1) / tile;
    const int64_t tile_min = (T.tile_min > 0 && nrtiles >= 2)
                                 ? std::max<int64_t>((int64_t)T.tile_min * nrtiles, (int64_t)T.seg + 1)
                                 : INT64_MAX;
    const int64_t key_tiles = (int64_t)FM_XCDS * (maxpos + 1);
    if (key_tiles + nrtiles >= (1LL << 32)) return fm_fail(m, FM_ERANGE, "too many row tiles");
    FM_HIP(m, hipMemsetAsync(out->long_first, 0, (size_t)(nlong + 1) * sizeof(int64_t), st));
    hipLaunchKernelGGL(k_full_items, dim3((unsigned)nlong), dim3(256), 0, st, (const int64_t*)m->colptr,
                       (const int32_t*)m->crow, (const int32_t*)out->long_col, m->N, T.seg, panel, heavy_min,
                       maxpos, tile, tile_min, T.tile_seg, 0, out->long_first, (const int64_t*)nullptr, (int32_t*)nullptr, (int64_t*)nullptr,
                       (int32_t*)nullptr, (uint32_t*)nullptr);
    FM_HIP(m, hipGetLastError());
    FM_TRY(fm_scan_exclusive_i64(m, out->long_first, nlong + 1, st));
    std::vector<int64_t> h_first((size_t)nlong + 1);
    FM_HIP(m, hipMemcpyAsync(h_first.data(), out->long_first, (size_t)(nlong + 1) * sizeof(int64_t),
                             hipMemcpyDeviceToHost, st));
    FM_HIP(m, hipStreamSynchronize(st));
    const int64_t nitems = h_first[(size_t)nlong];
    if (nitems >= (1LL << 32)) return fm_fail(m, FM_ERANGE, "too many column items");
    FM_TRY(fm_dev_alloc(m, (void**)&out->item_col, (size_t)nitems * sizeof(int32_t)));
    FM_TRY(fm_dev_alloc(m, (void**)&out->item_beg, (size_t)nitems * sizeof(int64_t)));
    FM_TRY(fm_dev_alloc(m, (void**)&out->item_len, (size_t)nitems * sizeof(int32_t)));
    uint32_t *k0 = nullptr, *i0 = nullptr, *k1 = nullptr, *i1 = nullptr;
    FM_TRY(fm_dev_alloc(m, (void**)&k0, (size_t)nitems * 4));
    FM_TRY(fm_dev_alloc(m, (void**)&i0, (size_t)nitems * 4));
    FM_TRY(fm_dev_alloc(m, (void**)&k1, (size_t)nitems * 4));
    FM_TRY(fm_dev_alloc(m, (void**)&i1, (size_t)nitems * 4));
    hipLaunchKernelGGL(k_full_items, dim3((unsigned)nlong), dim3(256), 0, st, (const int64_t*)m->colptr,
                       (const int32_t*)m->crow, (const int32_t*)out->long_col, m->N, T.seg, panel, heavy_min,
                       maxpos, tile, tile_min, T.tile_seg, 1, (int64_t*)nullptr, (const int64_t*)out->long_first, out->item_col, out->item_beg,
                       out->item_len, k0);
    FM_HIP(m, hipGetLastError());
    // 3. processing order: stable sort of the item ids by (XCD list, panel position)
    hipLaunchKernelGGL(k_iota_u32, dim3(blocks_for(nitems, 256)), dim3(256), 0, st, i0, nitems);
    FM_HIP(m, hipGetLastError());
    bool alt = false;
    FM_TRY(fm_sort_by_key_u32(m, k0, i0, k1, i1, nitems, bits_for(key_tiles + nrtiles), st, &alt));
    int64_t* d_off = nullptr;
    FM_TRY(fm_dev_alloc(m, (void**)&d_off, (2 * FM_XCDS + 1) * sizeof(int64_t)));
    hipLaunchKernelGGL(k_list_offsets, dim3(1), dim3(64), 0, st, (const uint32_t*)(alt ? k1 : k0), nitems, maxpos, d_off);
    FM_HIP(m, hipGetLastError());
    int64_t h_off[2 * FM_XCDS + 1];
    FM_HIP(m, hipMemcpyAsync(h_off, d_off, sizeof(h_off), hipMemcpyDeviceToHost, st));
    FM_HIP(m, hipStreamSynchronize(st));
    for (int x = 0; x <= FM_XCDS; ++x) out->list_off[x] = h_off[x];
    for (int x = 0; x < FM_XCDS; ++x) out->list_mid[x] = h_off[FM_XCDS + 1 + x];
    out->tile_rows = tile;
    out->ntiles = 0;
    if (out->list_off[FM_XCDS] < nitems) {  // there are tile items
        out->ntiles = nrtiles;
        FM_TRY(fm_dev_alloc(m, (void**)&out->tile_ptr, (size_t)(nrtiles + 1) * sizeof(int64_t)));
        hipLaunchKernelGGL(k_tile_ptr, dim3(blocks_for(nrtiles + 1, 256)), dim3(256), 0, st,
                           (const uint32_t*)(alt ? k1 : k0), nitems, key_tiles, nrtiles, out->tile_ptr);
        FM_HIP(m, hipGetLastError());
        FM_HIP(m, hipStreamSynchronize(st));
    }
    out->order = alt ? i1 : i0;
    fm_dev_free(m, alt ? i0 : i1);
    FM_TRY(fm_dev_alloc(m, (void**)&out->ord_beg, (size_t)nitems * sizeof(int64_t)));
    FM_TRY(fm_dev_alloc(m, (void**)&out->ord_len, (size_t)nitems * sizeof(int32_t)));
    hipLaunchKernelGGL(k_order_items, dim3(blocks_for(nitems, 256)), dim3(256), 0, st, (const uint32_t*)out->order,
                       nitems, (const int64_t*)out->item_beg, (const int32_t*)out->item_len, out->ord_beg,
                       out->ord_len);
    FM_HIP(m, hipGetLastError());
    FM_HIP(m, hipStreamSynchronize(st));
    fm_dev_free(m, k0);
    fm_dev_free(m, k1);
    fm_dev_free(m, d_off);
    // 4. columns with very many items get a workgroup each in the finish step
    std::vector<int32_t> h_vlong;
    for (int64_t lc = 0; lc < nlong; ++lc)
        if (h_first[(size_t)lc + 1] - h_first[(size_t)lc] > T.vlong) h_vlong.push_back((int32_t)lc);
    out->nvlong = (int64_t)h_vlong.size();
    if (out->nvlong > 0) {
        FM_TRY(fm_dev_alloc(m, (void**)&out->vlong, h_vlong.size() * sizeof(int32_t)));
        FM_HIP(m, hipMemcpy(out->vlong, h_vlong.data(), h_vlong.size() * sizeof(int32_t), hipMemcpyHostToDevice));
    }
    out->nlong = nlong;
    out->nitems = nitems;
    out->h_long_off[1] = nlong;
    out->h_item_off[1] = nitems;
    fm_dev_free(m, vcol);
    fm_dev_free(m, tl);
    fm_dev_free(m, ti);
    return FM_OK;
}

extern "C" int fm_build_csc(fm_matrix* m, void* hip_stream)
{
    if (m == nullptr) return FM_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    if (m->has_csc) return FM_OK;
    const int64_t n = m->nnz;
    FM_TRY(fm_dev_alloc(m, (void**)&m->colptr, (size_t)(m->D + 1) * sizeof(int64_t)));
    FM_TRY(fm_dev_alloc(m, (void**)&m->crow, (size_t)(n > 0 ? n : 1) * sizeof(int32_t)));
    FM_TRY(fm_dev_alloc(m, (void**)&m->cval, (size_t)(n > 0 ? n : 1) * sizeof(float)));
    if (n == 0) {
        FM_HIP(m, hipMemsetAsync(m->colptr, 0, (size_t)(m->D + 1) * sizeof(int64_t), st));
    } else {
        uint32_t *k0 = nullptr, *i0 = nullptr, *k1 = nullptr, *i1 = nullptr;
        FM_TRY(fm_dev_alloc(m, (void**)&k0, (size_t)n * 4));
        FM_TRY(fm_dev_alloc(m, (void**)&i0, (size_t)n * 4));
        FM_TRY(fm_dev_alloc(m, (void**)&k1, (size_t)n * 4));
        FM_TRY(fm_dev_alloc(m, (void**)&i1, (size_t)n * 4));
        hipLaunchKernelGGL(k_init_keys, dim3(blocks_for(n, 256)), dim3(256), 0, st, (const int32_t*)m->col, k0, i0, n);
        FM_HIP(m, hipGetLastError());
        bool alt = false;
        FM_TRY(fm_sort_by_key_u32(m, k0, i0, k1, i1, n, bits_for(m->D - 1), st, &alt));
        const uint32_t* sk = alt ? k1 : k0;
        const uint32_t* perm = alt ? i1 : i0;
        hipLaunchKernelGGL(k_gather_transposed, dim3(blocks_for(n, 256)), dim3(256), 0, st, perm,
                           (const int64_t*)m->rowptr, m->N, (const float*)m->val, m->crow, m->cval, n);
        FM_HIP(m, hipGetLastError());
        hipLaunchKernelGGL(k_ptr_from_sorted, dim3(blocks_for(m->D + 1, 256)), dim3(256), 0, st, sk, n, m->D,
                           m->colptr);
        FM_HIP(m, hipGetLastError());
        FM_HIP(m, hipStreamSynchronize(st));
        fm_dev_free(m, k0);
        fm_dev_free(m, i0);
        fm_dev_free(m, k1);
        fm_dev_free(m, i1);
    }
    FM_TRY(fm_build_full_index(m, 0, st));
    FM_TRY(fm_dense_build_index(m, st));  // nothing unless every row stores all columns
    FM_HIP(m, hipStreamSynchronize(st));
    m->has_csc = true;
    fm_drop_workspace(m);
    return FM_OK;
}

static int partition_impl(fm_matrix* m, int32_t P, const int32_t* place, hipStream_t st);

// One orientation of the per-stratum matrices: the entries in (stratum, major, minor) order, the list
// of the (stratum, major) pairs that hold an entry with the offset of their first one, and where every
// stratum starts in the entries (h_ent_off) and in that list (h_list_off).
// (batches: the column orientation keyed by row block alone, P = number of batches)
struct StrataSide {
    int32_t* ind = nullptr;
    float* val = nullptr;
    int32_t* nz_major = nullptr;
    int64_t* nz_beg = nullptr;  // [count + 1]
    int64_t count = 0;
    std::vector<int64_t> h_ent_off, h_list_off;  // [P + 1]
};

static int build_strata_side(fm_matrix* m, bool by_rows, hipStream_t st, StrataSide* out, int32_t P, bool batches = false)
{
    const int64_t n = m->nnz;
    const int64_t nmajor = by_rows ? m->N : m->D;
    const int64_t* major = by_rows ? m->rowptr : m->colptr;
    const int32_t* minor = by_rows ? m->col : m->crow;
    const float* val = by_rows ? m->val : m->cval;
    out->h_ent_off.assign(P + 1, 0);
    out->h_list_off.assign(P + 1, 0);
    FM_TRY(fm_dev_alloc(m, (void**)&out->ind, (size_t)(n > 0 ? n : 1) * sizeof(int32_t)));
    FM_TRY(fm_dev_alloc(m, (void**)&out->val, (size_t)(n > 0 ? n : 1) * sizeof(float)));
    if (n == 0) {
        FM_TRY(fm_dev_alloc(m, (void**)&out->nz_major, sizeof(int32_t)));
        FM_TRY(fm_dev_alloc(m, (void**)&out->nz_beg, sizeof(int64_t)));
        FM_HIP(m, hipMemsetAsync(out->nz_beg, 0, sizeof(int64_t), st));
        return FM_OK;
    }
    uint32_t *k0 = nullptr, *i0 = nullptr, *k1 = nullptr, *i1 = nullptr;
    FM_TRY(fm_dev_alloc(m, (void**)&k0, (size_t)n * 4));
    FM_TRY(fm_dev_alloc(m, (void**)&i0, (size_t)n * 4));
    FM_TRY(fm_dev_alloc(m, (void**)&k1, (size_t)n * 4));
    FM_TRY(fm_dev_alloc(m, (void**)&i1, (size_t)n * 4));
    hipLaunchKernelGGL(k_stratum_keys, dim3(blocks_for(n, 256)), dim3(256), 0, st, major, nmajor, minor, n, m->N,
                       m->D, P, batches ? 2 : (by_rows ? 1 : 0), batches ? nullptr : (const int32_t*)m->d_place, k0, i0);
    FM_HIP(m, hipGetLastError());
    bool alt = false;
    FM_TRY(fm_sort_by_key_u32(m, k0, i0, k1, i1, n, bits_for(P - 1), st, &alt));
    const uint32_t* keys = alt ? k1 : k0;
    const uint32_t* perm = alt ? i1 : i0;
    hipLaunchKernelGGL(k_gather_pairs, dim3(blocks_for(n, 256)), dim3(256), 0, st, perm, minor, val, out->ind, out->val, n);
    FM_HIP(m, hipGetLastError());
    // the stable sort keeps the entries of a stratum in the order of the source (by major index): the
    // (stratum, major) pairs are runs, found by comparing neighbours
    int32_t* maj = reinterpret_cast<int32_t*>(alt ? k0 : k1);  // the buffer the sort no longer needs
    hipLaunchKernelGGL(k_major_of, dim3(blocks_for(n, 256)), dim3(256), 0, st, perm, major, nmajor, maj, n);
    FM_HIP(m, hipGetLastError());
    int64_t* pos = nullptr;
    FM_TRY(fm_dev_alloc(m, (void**)&pos, (size_t)(n + 1) * sizeof(int64_t)));
    hipLaunchKernelGGL(k_head_flags, dim3(blocks_for(n, 256)), dim3(256), 0, st, keys, (const int32_t*)maj, n, pos);
    FM_HIP(m, hipGetLastError());
    FM_HIP(m, hipMemsetAsync(pos + n, 0, sizeof(int64_t), st));
    FM_TRY(fm_scan_exclusive_i64(m, pos, n + 1, st));
    int64_t count = 0;
    FM_HIP(m, hipMemcpyAsync(&count, pos + n, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    FM_HIP(m, hipStreamSynchronize(st));
    out->count = count;
    FM_TRY(fm_dev_alloc(m, (void**)&out->nz_major, (size_t)count * sizeof(int32_t)));
    FM_TRY(fm_dev_alloc(m, (void**)&out->nz_beg, (size_t)(count + 1) * sizeof(int64_t)));
    hipLaunchKernelGGL(k_compact_heads, dim3(blocks_for(n, 256)), dim3(256), 0, st, keys, (const int32_t*)maj,
                       (const int64_t*)pos, n, out->nz_major, out->nz_beg);
    FM_HIP(m, hipGetLastError());
    FM_HIP(m, hipMemcpyAsync(out->nz_beg + count, &n, sizeof(int64_t), hipMemcpyHostToDevice, st));
    // where every stratum starts: in the entries (keys smaller than s), then in the list of pairs
    int64_t *d_ent = nullptr, *d_list = nullptr;
    FM_TRY(fm_dev_alloc(m, (void**)&d_ent, (size_t)(P + 1) * sizeof(int64_t)));
    FM_TRY(fm_dev_alloc(m, (void**)&d_list, (size_t)(P + 1) * sizeof(int64_t)));
    hipLaunchKernelGGL(k_ptr_from_sorted, dim3(blocks_for(P + 1, 256)), dim3(256), 0, st, keys, n, (int64_t)P, d_ent);
    FM_HIP(m, hipGetLastError());
    hipLaunchKernelGGL(k_lower_bounds, dim3(blocks_for(P + 1, 256)), dim3(256), 0, st, (const int64_t*)out->nz_beg, count,
                       (const int64_t*)d_ent, (int64_t)(P + 1), d_list);
    FM_HIP(m, hipGetLastError());
    FM_HIP(m, hipMemcpyAsync(out->h_ent_off.data(), d_ent, (size_t)(P + 1) * sizeof(int64_t), hipMemcpyDeviceToHost, st));
    FM_HIP(m, hipMemcpyAsync(out->h_list_off.data(), d_list, (size_t)(P + 1) * sizeof(int64_t), hipMemcpyDeviceToHost, st));
    FM_HIP(m, hipStreamSynchronize(st));
    for (void* q : {(void*)k0, (void*)i0, (void*)k1, (void*)i1, (void*)pos, (void*)d_ent, (void*)d_list}) fm_dev_free(m, q);
    return FM_OK;
}

extern "C" int fm_partition(fm_matrix* m, int32_t P, void* hip_stream)
{
    if (m == nullptr) return FM_EINVAL;
    return partition_impl(m, P, nullptr, (hipStream_t)hip_stream);
}

extern "C" int fm_partition_placed(fm_matrix* m, int32_t P, const int32_t* place, void* hip_stream)
{
    if (m == nullptr) return FM_EINVAL;
    if (place == nullptr) return fm_fail(m, FM_EINVAL, "place is NULL");
    for (int64_t j = 0; j < m->D; ++j)
        if (place[j] < 0 || place[j] >= P)
            return fm_fail(m, FM_ERANGE, "place[%lld] = %d outside [0,%d)", (long long)j, place[j], P);
    return partition_impl(m, P, place, (hipStream_t)hip_stream);
}

static int partition_impl(fm_matrix* m, int32_t P, const int32_t* place, hipStream_t st)
{
    if (!m->has_csc) return fm_fail(m, FM_ESTATE, "fm_partition needs fm_build_csc first");
    if (P < 1 || P > FM_MAXP) return fm_fail(m, FM_EINVAL, "P=%d outside 1..%d", P, FM_MAXP);
    if (m->P != 0) return fm_fail(m, FM_ESTATE, "matrix is already partitioned (P=%d)", m->P);
    if (m->N < 1 || m->D < 1) return fm_fail(m, FM_EINVAL, "cannot partition an empty matrix");
    m->P = P;
    m->h_rb.resize(P + 1);
    m->h_cb.resize(P + 1);
    for (int32_t b = 0; b <= P; ++b) {
        m->h_rb[b] = (int64_t)(((__int128)b * (__int128)m->N) / (__int128)P);
        m->h_cb[b] = (int64_t)(((__int128)b * (__int128)m->D) / (__int128)P);
    }
    std::vector<float> h_rho((size_t)P);
    for (int32_t b = 0; b < P; ++b) h_rho[b] = (float)((double)(m->h_rb[b + 1] - m->h_rb[b]) / (double)m->N);
    FM_TRY(fm_dev_alloc(m, (void**)&m->d_rho, (size_t)P * sizeof(float)));
    FM_HIP(m, hipMemcpy(m->d_rho, h_rho.data(), (size_t)P * sizeof(float), hipMemcpyHostToDevice));
    FM_TRY(fm_dev_alloc(m, (void**)&m->d_rb, (size_t)(P + 1) * sizeof(int64_t)));
    FM_HIP(m, hipMemcpy(m->d_rb, m->h_rb.data(), (size_t)(P + 1) * sizeof(int64_t), hipMemcpyHostToDevice));
    FM_TRY(fm_ensure_lazy(m));
    if (place != nullptr) {
        FM_TRY(fm_dev_alloc(m, (void**)&m->d_place, (size_t)m->D * sizeof(int32_t)));
        FM_HIP(m, hipMemcpy(m->d_place, place, (size_t)m->D * sizeof(int32_t), hipMemcpyHostToDevice));
    }
    FM_TRY(fm_dev_alloc(m, (void**)&m->col_mark, (size_t)m->D * sizeof(int32_t)));
    FM_HIP(m, hipMemsetAsync(m->col_mark, 0, (size_t)m->D * sizeof(int32_t), st));

    StrataSide rows, cols;
    FM_TRY(build_strata_side(m, true, st, &rows, P));
    FM_TRY(build_strata_side(m, false, st, &cols, P));
    m->s_col = rows.ind;
    m->s_val = rows.val;
    // the rows that have an entry in stratum s: its refresh visits only these (a row's entries end
    // where those of the next listed row begin)
    m->s_touched = rows.nz_major;
    m->s_touched_beg = rows.nz_beg;
    m->ntouched = rows.count;
    m->h_touch_off = rows.h_list_off;
    m->s_row = cols.ind;
    m->s_cval = cols.val;
    m->s_ncol = cols.nz_major;
    m->s_ncol_beg = cols.nz_beg;
    m->nncol = cols.count;
    m->h_ncol_off = cols.h_list_off;
    m->h_strat_nnz_off = cols.h_ent_off;

    // cell table (row block, column block or worker the column started at), counted entry by entry
    m->h_cell_nnz.clear();
    if (P <= FM_MAXP_CELLS) {
        m->h_cell_nnz.assign((size_t)P * P, 0);
        unsigned long long* d_cell = nullptr;
        FM_TRY(fm_dev_alloc(m, (void**)&d_cell, (size_t)P * P * sizeof(unsigned long long)));
        FM_HIP(m, hipMemsetAsync(d_cell, 0, (size_t)P * P * sizeof(unsigned long long), st));
        if (m->nnz > 0) {
            hipLaunchKernelGGL(k_cell_count, dim3(blocks_for(m->nnz, 256)), dim3(256), 0, st, (const int64_t*)m->rowptr,
                               m->N, (const int32_t*)m->col, m->nnz, m->D, (const int32_t*)m->d_place, P, d_cell);
            FM_HIP(m, hipGetLastError());
        }
        FM_HIP(m, hipMemcpyAsync(m->h_cell_nnz.data(), d_cell, (size_t)P * P * sizeof(int64_t), hipMemcpyDeviceToHost, st));
        FM_HIP(m, hipStreamSynchronize(st));
        fm_dev_free(m, d_cell);
    }
    FM_TRY(fm_build_long_index(m, m->s_ncol_beg, m->s_ncol, m->nncol, m->h_ncol_off, P, &m->lstrat, st));
    FM_HIP(m, hipStreamSynchronize(st));
    fm_drop_workspace(m);
    return FM_OK;
}

int fm_ensure_lazy(fm_matrix* m)
{
    if (m->lazy_last != nullptr) return FM_OK;
    return fm_dev_alloc(m, (void**)&m->lazy_last, (size_t)std::max<int64_t>(m->D, 1) * sizeof(int32_t));
}

extern "C" int fm_partition_batches(fm_matrix* m, int32_t B, void* hip_stream)
{
    if (m == nullptr) return FM_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    if (!m->has_csc) return fm_fail(m, FM_ESTATE, "fm_partition_batches needs fm_build_csc first");
    if (B < 1 || B > FM_MAXP) return fm_fail(m, FM_EINVAL, "B=%d outside 1..%d", B, FM_MAXP);
    if (m->B != 0) return fm_fail(m, FM_ESTATE, "row batches are already built (B=%d)", m->B);
    if (m->N < 1 || m->D < 1) return fm_fail(m, FM_EINVAL, "cannot split an empty matrix");
    m->B = B;
    m->h_bb.resize(B + 1);
    std::vector<float> h_rho((size_t)B);
    for (int32_t b = 0; b <= B; ++b) m->h_bb[b] = (int64_t)(((__int128)b * (__int128)m->N) / (__int128)B);
    for (int32_t b = 0; b < B; ++b) h_rho[b] = (float)((double)(m->h_bb[b + 1] - m->h_bb[b]) / (double)m->N);
    FM_TRY(fm_dev_alloc(m, (void**)&m->d_brho, (size_t)B * sizeof(float)));
    FM_HIP(m, hipMemcpy(m->d_brho, h_rho.data(), (size_t)B * sizeof(float), hipMemcpyHostToDevice));
    FM_TRY(fm_dev_alloc(m, (void**)&m->d_bb, (size_t)(B + 1) * sizeof(int64_t)));
    FM_HIP(m, hipMemcpy(m->d_bb, m->h_bb.data(), (size_t)(B + 1) * sizeof(int64_t), hipMemcpyHostToDevice));
    FM_TRY(fm_ensure_lazy(m));
    if (m->col_mark == nullptr) {
        FM_TRY(fm_dev_alloc(m, (void**)&m->col_mark, (size_t)m->D * sizeof(int32_t)));
        FM_HIP(m, hipMemsetAsync(m->col_mark, 0, (size_t)m->D * sizeof(int32_t), st));
    }
    StrataSide cols;
    FM_TRY(build_strata_side(m, false, st, &cols, B, true));
    m->b_row = cols.ind;
    m->b_cval = cols.val;
    m->b_ncol = cols.nz_major;
    m->b_ncol_beg = cols.nz_beg;
    m->nbcol = cols.count;
    m->h_bcol_off = cols.h_list_off;
    m->h_batch_nnz_off = cols.h_ent_off;
    FM_TRY(fm_build_long_index(m, m->b_ncol_beg, m->b_ncol, m->nbcol, m->h_bcol_off, B, &m->lbatch, st));
    FM_HIP(m, hipStreamSynchronize(st));
    fm_drop_workspace(m);
    return FM_OK;
}
