// On-GPU reconstruction of a snapshot from the previous one and a graph difference
// (Section "Graph-difference Based Input Transfer"): common = A_prev \ deleted,
// A_next = common U added, both kept as CSR of A + I with ascending duplicate-free rows.
//
// Because both difference lists arrive sorted by (row, col), no global prefix scan is needed:
//   rowptr_next[r] = rowptr_prev[r] + #added with row < r - #deleted with row < r
// and "#entries with row < r" is a lower bound in a sorted list.  Every tile is independent:
//   1. rowptr_kernel  (tiles of rows)         new row pointers, dinv = (row length)^(-1/2),
//                                             and add_ptr[r] = #added with row < r (workspace);
//   2. merge_kernel   (tiles of old entries)  every old entry finds its new position
//        pos = rowptr_next[r] + (i - rowptr_prev[r]) - #deleted in row with col < c
//                                                    + #added   in row with col < c
//      and writes itself there unless deleted; the added entries that fall between an old entry
//      and its predecessor in the row are written by that old entry's lane.  Tiles hold equal
//      numbers of old entries, so hub rows of power-law graphs are spread over many workgroups,
//      and untouched rows cost one coalesced read and one coalesced write per entry.
#include "common.hpp"

namespace {

using namespace dgnn;

constexpr int kRowThreads = 256;
constexpr int kRowsPerThread = 4;
constexpr int kRowTile = kRowThreads * kRowsPerThread;

constexpr int kMergeThreads = 256;
constexpr int kMergeItems = 4;
constexpr int kMergeTile = kMergeThreads * kMergeItems;

__device__ __forceinline__ void report(int32_t *status, int code) {
    if (!status) return;
    int old = *status;
    while (old == 0 || code < old) {
        int seen = atomicCAS(status, old, code);
        if (seen == old) break;
        old = seen;
    }
}

// Per-row counts of a sorted row list restricted to [lo, hi), accumulated into LDS counters by
// run boundaries: the last element of a run adds (j + 1), the first subtracts j.
__device__ __forceinline__ void count_runs(const int32_t *__restrict__ rows, int lo, int hi, int r0, int nr,
                                           int *cnt, int tid) {
    for (int j = lo + tid; j < hi; j += kRowThreads) {
        int r = rows[j];
        bool first = (j == lo) || rows[j - 1] != r;
        bool last = (j == hi - 1) || rows[j + 1] != r;
        unsigned k = (unsigned)(r - r0);
        if (k < (unsigned)nr) {
            if (last) atomicAdd(&cnt[k], j + 1);
            if (first) atomicSub(&cnt[k], j);
        }
    }
}

__global__ __launch_bounds__(kRowThreads) void rowptr_kernel(
    int n, const int32_t *__restrict__ rowptr_prev,
    const int32_t *__restrict__ add_row, int n_add, const int32_t *__restrict__ del_row, int n_del,
    int32_t *__restrict__ rowptr_next, int32_t *__restrict__ add_ptr, float *__restrict__ dinv,
    int32_t *status) {
    __shared__ int s_add[kRowTile];
    __shared__ int s_del[kRowTile];
    __shared__ int s_bound[4];
    __shared__ int s_wsum[2][kRowThreads / kWave];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int r0 = blockIdx.x * kRowTile;
    const int r1 = min(r0 + kRowTile, n);
    const int nr = r1 - r0;

    if (blockIdx.x == 0 && tid == 0 && status) *status = 0;
    if (tid < 4) {
        const int32_t *list = tid < 2 ? add_row : del_row;
        int len = tid < 2 ? n_add : n_del;
        s_bound[tid] = lower_bound(list, 0, len, (tid & 1) ? r1 : r0);
    }
    for (int i = tid; i < kRowTile; i += kRowThreads) { s_add[i] = 0; s_del[i] = 0; }
    __syncthreads();
    const int a0 = s_bound[0], a1 = s_bound[1], d0 = s_bound[2], d1 = s_bound[3];
    count_runs(add_row, a0, a1, r0, nr, s_add, tid);
    count_runs(del_row, d0, d1, r0, nr, s_del, tid);
    __syncthreads();

    int ca[kRowsPerThread], cd[kRowsPerThread];
    int sa = 0, sd = 0;
#pragma unroll
    for (int k = 0; k < kRowsPerThread; ++k) {
        ca[k] = s_add[tid * kRowsPerThread + k];
        cd[k] = s_del[tid * kRowsPerThread + k];
        sa += ca[k];
        sd += cd[k];
    }
    int ia = wave_scan_add(sa, lane), id = wave_scan_add(sd, lane);
    if (lane == kWave - 1) { s_wsum[0][wave] = ia; s_wsum[1][wave] = id; }
    __syncthreads();
    int oa = a0 + ia - sa, od = d0 + id - sd;      // exclusive offsets of this thread's first row
    for (int w = 0; w < wave; ++w) { oa += s_wsum[0][w]; od += s_wsum[1][w]; }

#pragma unroll
    for (int k = 0; k < kRowsPerThread; ++k) {
        int r = r0 + tid * kRowsPerThread + k;
        if (r < r1) {
            int rp = rowptr_prev[r], rq = rowptr_prev[r + 1];
            rowptr_next[r] = rp + oa - od;
            add_ptr[r] = oa;
            if (dinv) dinv[r] = 1.0f / sqrtf((float)(rq - rp + ca[k] - cd[k]));
        }
        oa += ca[k];
        od += cd[k];
    }
    if (r1 == n && tid == 0) {
        rowptr_next[n] = rowptr_prev[n] + n_add - n_del;
        add_ptr[n] = n_add;
    }
}

__global__ __launch_bounds__(kMergeThreads) void merge_kernel(
    int n, const int32_t *__restrict__ rowptr_prev, const int32_t *__restrict__ colidx_prev, int nnz_prev,
    const int32_t *__restrict__ add_col, int n_add, const int32_t *__restrict__ del_col, int n_del,
    const int32_t *__restrict__ rowptr_next, const int32_t *__restrict__ add_ptr,
    int32_t *__restrict__ colidx_next, int cap_next, int32_t *status) {
    __shared__ int s_rowid[kMergeTile];
    __shared__ int s_la[kMergeTile];
    __shared__ int s_rp[kMergeTile + 2];
    __shared__ int s_rn[kMergeTile + 2];
    __shared__ int s_ap[kMergeTile + 2];
    __shared__ int s_rows[2];
    __shared__ int s_wmax[kMergeThreads / kWave];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int i0 = (int)((int64_t)blockIdx.x * kMergeTile);
    const int i1 = (int)min((int64_t)i0 + kMergeTile, (int64_t)nnz_prev);
    const int cnt = i1 - i0;

    if (wave < 2) {   // the rows that hold the first and the last entry of the tile, one wavefront each
        int r = wave_find_row(rowptr_prev, n, wave == 0 ? i0 : i1 - 1, lane);
        if (lane == 0) s_rows[wave] = max(r, 0);
    }
    for (int p = tid; p < kMergeTile; p += kMergeThreads) s_rowid[p] = 0;
    __syncthreads();
    const int r_first = s_rows[0];
    const int nr = s_rows[1] - r_first + 1;
    if (nr > kMergeTile || nr < 1) {   // only possible when A_prev has empty rows
        if (tid == 0) report(status, DGNN_BAD_EMPTY_ROW);
        return;
    }
    for (int k = tid; k <= nr; k += kMergeThreads) {
        int r = r_first + k;
        s_rp[k] = rowptr_prev[r];
        s_rn[k] = rowptr_next[r];
        s_ap[k] = add_ptr[r];
    }
    __syncthreads();
    for (int k = tid + 1; k < nr; k += kMergeThreads) {   // rows that start inside the tile
        unsigned p = (unsigned)(s_rp[k] - i0);
        if (p < (unsigned)cnt) atomicMax(&s_rowid[p], k);
    }
    __syncthreads();
    {   // inclusive max-scan turns the row heads into a row id per entry
        int v[kMergeItems];
        int m = 0;
#pragma unroll
        for (int k = 0; k < kMergeItems; ++k) {
            m = max(m, s_rowid[tid * kMergeItems + k]);
            v[k] = m;
        }
        int inc = wave_scan_max(m, lane);
        if (lane == kWave - 1) s_wmax[wave] = inc;
        int before = __shfl_up(inc, 1, kWave);
        if (lane == 0) before = 0;
        __syncthreads();
        for (int w = 0; w < wave; ++w) before = max(before, s_wmax[w]);
#pragma unroll
        for (int k = 0; k < kMergeItems; ++k) s_rowid[tid * kMergeItems + k] = max(v[k], before);
    }
    __syncthreads();

    int c_[kMergeItems], ld_[kMergeItems], la_[kMergeItems];
    bool dead_[kMergeItems];
#pragma unroll
    for (int k = 0; k < kMergeItems; ++k) {
        const int p = tid + k * kMergeThreads;
        c_[k] = 0; ld_[k] = 0; la_[k] = 0; dead_[k] = false;
        if (p < cnt) {
            const int rr = s_rowid[p];
            const int as = s_ap[rr], ae = s_ap[rr + 1];
            const int ds = s_rp[rr] + as - s_rn[rr];
            const int de = s_rp[rr + 1] + ae - s_rn[rr + 1];
            const int c = colidx_prev[i0 + p];
            c_[k] = c;
            if (as >= 0 && as < ae && ae <= n_add) la_[k] = lower_bound(add_col, as, ae, c) - as;
            if (ds >= 0 && ds < de && de <= n_del) {
                int q = lower_bound(del_col, ds, de, c);
                ld_[k] = q - ds;
                dead_[k] = q < de && del_col[q] == c;
            }
            s_la[p] = la_[k];
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kMergeItems; ++k) {
        const int p = tid + k * kMergeThreads;
        if (p >= cnt) continue;
        const int i = i0 + p;
        const int rr = s_rowid[p];
        const int rp = s_rp[rr];
        const int as = s_ap[rr], ae = s_ap[rr + 1];
        const int base = s_rn[rr] + (i - rp) - ld_[k];
        if (as >= 0 && as < ae && ae <= n_add) {
            int j = 0;                                   // adds of the row that precede this entry's predecessor
            if (i > rp) j = p > 0 ? s_la[p - 1] : lower_bound(add_col, as, ae, colidx_prev[i - 1]) - as;
            for (; j < la_[k]; ++j) {
                unsigned pos = (unsigned)(base + j);
                if (pos < (unsigned)cap_next) colidx_next[pos] = add_col[as + j];
            }
            if (i == s_rp[rr + 1] - 1) {                 // last old entry of the row: the adds beyond it
                int jj = la_[k];
                if (as + jj < ae && add_col[as + jj] == c_[k]) ++jj;   // an "added" edge that already exists
                const int tail = base + (dead_[k] ? 0 : 1);
                for (; jj < ae - as; ++jj) {
                    unsigned pos = (unsigned)(tail + jj);
                    if (pos < (unsigned)cap_next) colidx_next[pos] = add_col[as + jj];
                }
            }
        }
        if (!dead_[k]) {
            unsigned pos = (unsigned)(base + la_[k]);
            if (pos < (unsigned)cap_next) colidx_next[pos] = c_[k];
        }
    }
}

// One thread per difference entry (added first, then deleted), then one per row of A_prev.
__global__ __launch_bounds__(256) void validate_kernel(
    int n, const int32_t *__restrict__ rowptr_prev, const int32_t *__restrict__ colidx_prev,
    const int32_t *__restrict__ add_row, const int32_t *__restrict__ add_col, int n_add,
    const int32_t *__restrict__ del_row, const int32_t *__restrict__ del_col, int n_del, int32_t *status) {
    int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= (int64_t)n_add + n_del) {
        int64_t r = g - n_add - n_del;
        if (r < n && rowptr_prev[r + 1] <= rowptr_prev[r]) report(status, DGNN_BAD_EMPTY_ROW);
        return;
    }
    const bool is_add = g < n_add;
    const int j = is_add ? (int)g : (int)(g - n_add);
    const int32_t *rows = is_add ? add_row : del_row;
    const int32_t *cols = is_add ? add_col : del_col;
    const int r = rows[j], c = cols[j];
    if (r < 0 || r >= n || c < 0 || c >= n) { report(status, DGNN_BAD_INDEX_RANGE); return; }
    if (j > 0) {
        int pr = rows[j - 1], pc = cols[j - 1];
        if (pr > r || (pr == r && pc >= c)) report(status, DGNN_BAD_DELTA_ORDER);
    }
    if (r == c) { report(status, DGNN_BAD_DIAGONAL); return; }
    int lo = rowptr_prev[r], hi = rowptr_prev[r + 1];
    if (lo < 0 || hi < lo) return;
    int q = lower_bound(colidx_prev, lo, hi, c);
    bool present = q < hi && colidx_prev[q] == c;
    if (is_add && present) report(status, DGNN_BAD_ADD_PRESENT);
    if (!is_add && !present) report(status, DGNN_BAD_DEL_ABSENT);
}

__global__ __launch_bounds__(256) void dinv_kernel(int n, const int32_t *__restrict__ rowptr, float *__restrict__ dinv) {
    int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r < n) dinv[r] = 1.0f / sqrtf((float)(rowptr[r + 1] - rowptr[r]));
}

}  // namespace

extern "C" const char *dgnn_strerror(int code) {
    switch (code) {
        case DGNN_OK: return "ok";
        case DGNN_ERR_NULL: return "a required pointer is NULL";
        case DGNN_ERR_SHAPE: return "bad size, feature width, window or dtype";
        case DGNN_ERR_CAPACITY: return "output buffer or workspace too small";
        case DGNN_ERR_OVERFLOW: return "n or nnz does not fit in int32";
        case DGNN_ERR_ALIAS: return "output aliases an input";
        case DGNN_ERR_HIP: return "HIP runtime error";
        case DGNN_ERR_ALIGN: return "feature pointer not 16-byte aligned";
        default: return "unknown dgnn status";
    }
}

extern "C" int dgnn_csr_dinv(int64_t n, const int32_t *rowptr, float *dinv, void *stream) {
    if (!rowptr || !dinv) return DGNN_ERR_NULL;
    if (n <= 0) return DGNN_ERR_SHAPE;
    if (!fits_i32(n)) return DGNN_ERR_OVERFLOW;
    hipLaunchKernelGGL(dinv_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       (int)n, rowptr, dinv);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

extern "C" int dgnn_delta_h2d(const int32_t *h_add_row, const int32_t *h_add_col, int64_t n_add,
                              const int32_t *h_del_row, const int32_t *h_del_col, int64_t n_del,
                              int32_t *d_add_row, int32_t *d_add_col, int32_t *d_del_row, int32_t *d_del_col,
                              void *stream) {
    if (n_add < 0 || n_del < 0) return DGNN_ERR_SHAPE;
    if (!fits_i32(n_add) || !fits_i32(n_del)) return DGNN_ERR_OVERFLOW;
    if (n_add > 0 && (!h_add_row || !h_add_col || !d_add_row || !d_add_col)) return DGNN_ERR_NULL;
    if (n_del > 0 && (!h_del_row || !h_del_col || !d_del_row || !d_del_col)) return DGNN_ERR_NULL;
    hipStream_t s = (hipStream_t)stream;
    const void *src[4] = {h_add_row, h_add_col, h_del_row, h_del_col};
    void *dst[4] = {d_add_row, d_add_col, d_del_row, d_del_col};
    const int64_t cnt[4] = {n_add, n_add, n_del, n_del};
    for (int k = 0; k < 4; ++k) {
        if (cnt[k] == 0) continue;
        if (hipMemcpyAsync(dst[k], src[k], (size_t)cnt[k] * sizeof(int32_t), hipMemcpyHostToDevice, s) != hipSuccess)
            return DGNN_ERR_HIP;
    }
    return DGNN_OK;
}

extern "C" int dgnn_delta_rebuild_workspace(int64_t n, int64_t nnz_prev, int64_t n_add, int64_t n_del, size_t *bytes) {
    if (!bytes) return DGNN_ERR_NULL;
    if (n <= 0 || nnz_prev < 0 || n_add < 0 || n_del < 0) return DGNN_ERR_SHAPE;
    if (!fits_i32(n + 1) || !fits_i32(nnz_prev + n_add)) return DGNN_ERR_OVERFLOW;
    *bytes = round_up((size_t)(n + 1) * sizeof(int32_t), 256);   // add_ptr
    return DGNN_OK;
}

extern "C" int dgnn_delta_rebuild(int64_t n,
                                  const int32_t *rowptr_prev, const int32_t *colidx_prev, int64_t nnz_prev,
                                  const int32_t *add_row, const int32_t *add_col, int64_t n_add,
                                  const int32_t *del_row, const int32_t *del_col, int64_t n_del,
                                  int32_t *rowptr_next, int32_t *colidx_next, int64_t cap_next, int64_t *nnz_next,
                                  float *dinv_next,
                                  void *ws, size_t ws_bytes, uint32_t flags, int32_t *d_status, void *stream) {
    if (!rowptr_prev || !colidx_prev || !rowptr_next || !colidx_next || !ws) return DGNN_ERR_NULL;
    if (n_add < 0 || n_del < 0) return DGNN_ERR_SHAPE;
    if (n_add > 0 && (!add_row || !add_col)) return DGNN_ERR_NULL;
    if (n_del > 0 && (!del_row || !del_col)) return DGNN_ERR_NULL;
    if (n <= 0 || nnz_prev <= 0 || (flags & ~DGNN_VALIDATE)) return DGNN_ERR_SHAPE;
    if (!fits_i32(n + 1) || !fits_i32(nnz_prev + n_add)) return DGNN_ERR_OVERFLOW;
    const int64_t nnz_new = nnz_prev + n_add - n_del;
    if (nnz_new < 0) return DGNN_ERR_SHAPE;
    if (cap_next < nnz_new) return DGNN_ERR_CAPACITY;
    size_t need = 0;
    int rc = dgnn_delta_rebuild_workspace(n, nnz_prev, n_add, n_del, &need);
    if (rc != DGNN_OK) return rc;
    if (ws_bytes < need) return DGNN_ERR_CAPACITY;
    if (rowptr_next == rowptr_prev || colidx_next == colidx_prev) return DGNN_ERR_ALIAS;
    if (nnz_next) *nnz_next = nnz_new;

    hipStream_t s = (hipStream_t)stream;
    int32_t *add_ptr = static_cast<int32_t *>(ws);
    const int cap = (int)min(cap_next, (int64_t)2147483647LL);

    hipLaunchKernelGGL(rowptr_kernel, dim3((unsigned)((n + kRowTile - 1) / kRowTile)), dim3(kRowThreads), 0, s,
                       (int)n, rowptr_prev, add_row, (int)n_add, del_row, (int)n_del, rowptr_next, add_ptr,
                       dinv_next, d_status);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    if ((flags & DGNN_VALIDATE) && d_status) {
        int64_t work = n_add + n_del + n;
        hipLaunchKernelGGL(validate_kernel, dim3((unsigned)((work + 255) / 256)), dim3(256), 0, s,
                           (int)n, rowptr_prev, colidx_prev, add_row, add_col, (int)n_add, del_row, del_col,
                           (int)n_del, d_status);
        DGNN_RETURN_IF_LAUNCH_FAILED();
    }
    hipLaunchKernelGGL(merge_kernel, dim3((unsigned)((nnz_prev + kMergeTile - 1) / kMergeTile)), dim3(kMergeThreads), 0, s,
                       (int)n, rowptr_prev, colidx_prev, (int)nnz_prev, add_col, (int)n_add, del_col, (int)n_del,
                       rowptr_next, add_ptr, colidx_next, cap, d_status);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}
