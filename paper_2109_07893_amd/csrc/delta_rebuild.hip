// On-GPU reconstruction of a snapshot from the previous one and a graph difference
// (Section "Graph-difference Based Input Transfer"): common = A_prev \ deleted,
// A_next = common U added, both kept as CSR of A + I with ascending duplicate-free rows.
//
// Because both difference lists arrive sorted by (row, col), no global prefix scan is needed:
//   rowptr_next[r] = rowptr_prev[r] + #added with row < r - #deleted with row < r
// and "#entries with row < r" is a lower bound in a sorted list.  Every tile is independent:
//   1. rowptr_kernel  (tiles of rows)         new row pointers, dinv = (row length)^(-1/2), and what the merge
//                                             has to know about the row in which each of its ranges begins
//                                             (in the workspace);
//   2. merge_kernel   (ranges of old entries) streams A_prev's column indices once: deleted entries
//      are struck out, added entries slotted in, a prefix sum per sub-tile gives the positions.
//      Ranges hold equal numbers of old entries, so hub rows of power-law graphs are spread over
//      many wavefronts, and an old entry costs one coalesced read and one coalesced write.
#include <algorithm>

#include "common.hpp"

namespace {

using namespace dgnn;

constexpr int kRowThreads = 256;
constexpr int kRowsPerThread = 4;          // rowptr_kernel moves a thread's rows as one 16-byte access: keep at 4
constexpr int kRowTile = kRowThreads * kRowsPerThread;
constexpr int kHeavyList = 16 * kRowTile;    // list entries per row tile beyond which counting walks no more

constexpr int kPerLane = 8;                  // old entries per lane and sub-tile of the merge
constexpr int kSub = kWave * kPerLane;       // old entries per sub-tile, at most
constexpr int kMaxRange = kSub * 16;         // old entries streamed by one wavefront, at most
constexpr int kTargetWaves = 16384;          // ranges shrink on small inputs so that about this many wavefronts exist

// The row in which a range of the merge begins: its extent in A_prev (rp, rp1) and in A_next (rn, rn1), and the stretch
// of the added list that belongs to it (as, ae); the deleted list's stretch follows from these.  us, ue: the row's
// stretch of the sorted value-update list of a weighted rebuild (0, 0 without one).
struct RangeStart { int rp, rp1, rn, rn1, as, ae, row, us, ue, pad; };

__device__ __forceinline__ void report(int32_t *status, int code) {
    if (!status) return;
    int old = *status;
    while (old == 0 || code < old) {
        int seen = atomicCAS(status, old, code);
        if (seen == old) break;
        old = seen;
    }
}

constexpr int kListPerThread = 4;           // consecutive list entries per thread and round of the walk below

// Per-row counts of a sorted row list restricted to [lo, hi), accumulated into LDS counters by
// run boundaries: the last element of a run adds (j + 1), the first subtracts j.
// A thread takes kListPerThread consecutive entries and their two neighbours, all loaded before any is looked at,
// so that a tile's usual stretch of a list costs one trip to memory.
__device__ __forceinline__ void count_runs(const int32_t *__restrict__ rows, int lo, int hi, int r0, int nr, int *cnt, int tid) {
#pragma unroll 1
    for (int base = lo; base < hi; base += kRowThreads * kListPerThread) {
        const int j0 = base + tid * kListPerThread;
        int r[kListPerThread + 2];        // rows[j0 - 1 .. j0 + kListPerThread]; -1 stands for "outside [lo, hi)"
#pragma unroll
        for (int k = 0; k < kListPerThread + 2; ++k) {
            const int j = j0 - 1 + k;
            r[k] = (j >= lo && j < hi) ? rows[j] : -1;
        }
#pragma unroll
        for (int k = 0; k < kListPerThread; ++k) {
            const int j = j0 + k;
            const unsigned q = (unsigned)(r[k + 1] - r0);
            if (j < hi && q < (unsigned)nr) {
                if (r[k + 2] != r[k + 1]) atomicAdd(&cnt[q], j + 1);     // last of its run
                if (r[k] != r[k + 1]) atomicSub(&cnt[q], j);             // first of its run
            }
        }
    }
}

// wave_find_row for two lists at once: the two searches advance in lock step, so their loads travel together.
// A list of length 0 (its pointer may be null) is not read and gives -1.
__device__ __forceinline__ void wave_find_row_pair(const int32_t *__restrict__ a, int na, int key_a, const int32_t *__restrict__ b,
                                                   int nb, int key_b, int lane, int &found_a, int &found_b) {
    int lo_a = 0, hi_a = na, lo_b = 0, hi_b = nb;
    while (hi_a > lo_a || hi_b > lo_b) {
        const int step_a = (hi_a - lo_a + kWave - 1) / kWave, step_b = (hi_b - lo_b + kWave - 1) / kWave;
        const int idx_a = lo_a + lane * step_a, idx_b = lo_b + lane * step_b;
        const bool in_a = hi_a > lo_a && idx_a < hi_a, in_b = hi_b > lo_b && idx_b < hi_b;
        const int v_a = in_a ? a[idx_a] : 0, v_b = in_b ? b[idx_b] : 0;
        const int m_a = __popcll(__ballot(in_a && v_a <= key_a)), m_b = __popcll(__ballot(in_b && v_b <= key_b));
        if (hi_a > lo_a) {
            if (m_a == 0) hi_a = lo_a;
            else { const int nlo = lo_a + (m_a - 1) * step_a + 1; hi_a = min(lo_a + m_a * step_a, hi_a); lo_a = nlo; }
        }
        if (hi_b > lo_b) {
            if (m_b == 0) hi_b = lo_b;
            else { const int nlo = lo_b + (m_b - 1) * step_b + 1; hi_b = min(lo_b + m_b * step_b, hi_b); lo_b = nlo; }
        }
    }
    found_a = lo_a - 1;
    found_b = lo_b - 1;
}

// The same counts from lower bounds: thread t finds where each of its rows begins inside [lo, hi),
// each search starting where the previous one ended.
__device__ __forceinline__ void count_by_search(const int32_t *__restrict__ rows, int lo, int hi, int r0, int nr,
                                                int *cnt, int tid) {
    int from = lo;
    int begin = 0;
#pragma unroll 1
    for (int k = 0; k <= kRowsPerThread; ++k) {
        const int t = tid * kRowsPerThread + k;
        if (t > nr) break;
        const int pos = lower_bound(rows, from, hi, r0 + t);     // first entry whose row is >= r0 + t
        if (k > 0) cnt[t - 1] = pos - begin;
        begin = pos;
        from = pos;
    }
}

// VEC: rowptr_prev, rowptr_next and dinv are 16-byte aligned, so a thread moves its four rows with one access each.
template <bool VEC>
__global__ __launch_bounds__(kRowThreads) void rowptr_kernel(
    int n, const int32_t *__restrict__ rowptr_prev,
    const int32_t *__restrict__ add_row, int n_add, const int32_t *__restrict__ del_row, int n_del,
    int32_t *__restrict__ rowptr_next, float *__restrict__ dinv,
    int range_len, int n_ranges, RangeStart *__restrict__ range_start,
    const int32_t *__restrict__ upd_row, int n_upd, int32_t *status) {
    __shared__ int s_add[kRowTile];
    __shared__ int s_del[kRowTile];
    __shared__ int s_bound[6];
    __shared__ int s_wsum[2][kRowThreads / kWave];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int r0 = blockIdx.x * kRowTile;
    const int r1 = min(r0 + kRowTile, n);
    const int nr = r1 - r0;
    const int r_own = r0 + tid * kRowsPerThread;          // this thread's rows: r_own .. r_own + 3
    const bool whole = r_own + kRowsPerThread <= n;       // all four exist

    if (blockIdx.x == 0 && tid == 0 && status) *status = 0;
    // the pointers of the thread's rows and the one after, on their way while the searches run
    int rp[kRowsPerThread + 1];
    if (VEC && whole) {
        const int4 v = *reinterpret_cast<const int4 *>(rowptr_prev + r_own);
        rp[0] = v.x; rp[1] = v.y; rp[2] = v.z; rp[3] = v.w;
        rp[4] = rowptr_prev[r_own + kRowsPerThread];
    } else {
#pragma unroll
        for (int k = 0; k <= kRowsPerThread; ++k) rp[k] = r_own + k <= n ? rowptr_prev[r_own + k] : 0;
    }
    {   // how many list entries have a row below r0 / below r1: one 64-ary search per wavefront and list; the
        // wavefronts that search the added list take the value-update list of a weighted rebuild along
        const int32_t *list = wave < 2 ? add_row : del_row;
        const int len = wave < 2 ? n_add : n_del;
        const int key = ((wave & 1) ? r1 : r0) - 1;
        int found, found_upd;
        wave_find_row_pair(list, len, key, upd_row, (wave < 2 && upd_row) ? n_upd : 0, key, lane, found, found_upd);
        if (lane == 0) {
            s_bound[wave] = found + 1;
            if (wave < 2) s_bound[4 + wave] = found_upd + 1;
        }
    }
    for (int i = tid; i < kRowTile; i += kRowThreads) { s_add[i] = 0; s_del[i] = 0; }
    __syncthreads();
    const int a0 = s_bound[0], a1 = s_bound[1], d0 = s_bound[2], d1 = s_bound[3];
    const int u0 = upd_row ? s_bound[4] : 0, u1 = upd_row ? s_bound[5] : 0;
    // A tile of hub rows can own a very long stretch of a list; walking it would leave the whole chip
    // waiting for this workgroup, so there the counts come from one lower bound per row instead.
    if (a1 - a0 <= kHeavyList) count_runs(add_row, a0, a1, r0, nr, s_add, tid);
    else count_by_search(add_row, a0, a1, r0, nr, s_add, tid);
    if (d1 - d0 <= kHeavyList) count_runs(del_row, d0, d1, r0, nr, s_del, tid);
    else count_by_search(del_row, d0, d1, r0, nr, s_del, tid);
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

    int rn[kRowsPerThread];
    float dv[kRowsPerThread];
#pragma unroll
    for (int k = 0; k < kRowsPerThread; ++k) {
        const int r = r_own + k;
        const int p = rp[k], q = rp[k + 1];
        rn[k] = p + oa - od;
        dv[k] = 1.0f / sqrtf((float)(q - p + ca[k] - cd[k]));
        if (r < r1) {
            // ranges of the merge that begin inside this row (few rows hold a multiple of the range length; a hub
            // row several): what the merge needs to know about the row, so that it starts without a search
            int us = -1, ue = 0;
            for (int g = max((p + range_len - 1) / range_len, 0); g < n_ranges && (int64_t)g * range_len < q; ++g) {
                if (upd_row && us < 0) {      // where the row's value updates lie: two searches inside the tile's stretch
                    us = lower_bound(upd_row, u0, u1, r);
                    ue = lower_bound(upd_row, us, u1, r + 1);
                }
                range_start[g] = RangeStart{p, q, p + oa - od, q + oa + ca[k] - od - cd[k], oa, oa + ca[k], r, max(us, 0), ue, 0};
            }
        }
        oa += ca[k];
        od += cd[k];
    }
    if (VEC && whole) {
        *reinterpret_cast<int4 *>(rowptr_next + r_own) = make_int4(rn[0], rn[1], rn[2], rn[3]);
        if (dinv) *reinterpret_cast<float4 *>(dinv + r_own) = make_float4(dv[0], dv[1], dv[2], dv[3]);
    } else {
#pragma unroll
        for (int k = 0; k < kRowsPerThread; ++k)
            if (r_own + k < r1) {
                rowptr_next[r_own + k] = rn[k];
                if (dinv) dinv[r_own + k] = dv[k];
            }
    }
    if (r1 == n && tid == 0) rowptr_next[n] = rowptr_prev[n] + n_add - n_del;
}

// First position in the ascending LDS array a[lo, hi) whose value is >= key (STRICT = false) or > key.
template <bool STRICT>
__device__ __forceinline__ int lds_bound(const int *a, int lo, int hi, int key) {
    while (lo < hi) {
        const int mid = lo + ((hi - lo) >> 1);
        const bool left = STRICT ? a[mid] <= key : a[mid] < key;
        if (left) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// One wavefront streams a contiguous range of old entries in sub-tiles of kSub entries.
// The work per OLD entry is a load, a position from a prefix sum, and a store; everything that
// needs a search is done per DIFFERENCE entry, of which there are few:
//   - the sub-tile's column indices are staged in LDS; each deleted entry that falls into the
//     sub-tile finds its old entry there by binary search and marks it dead, each added entry
//     finds the old entry it goes in front of (its slot) and counts itself there;
//   - where the row of a difference entry lies inside the sub-tile comes from the row pointers of A_prev, which
//     the wavefront streams beside the column indices: the pointers of the rows that meet the sub-tile (from the
//     row that holds its first entry on) are staged in LDS as well, fetched one sub-tile ahead like the column
//     indices, so a list entry (row, col) looks its row's extent up there and no load depends on another;
//   - both lists are consumed in order through two cursors, so the lists are never searched
//     (except once, where a range begins in the middle of a row); where a range's first row lies in A_prev,
//     in A_next and in the lists comes from rowptr_kernel;
//   - one prefix sum over (alive, added-before) gives every old entry and every slot its place
//     relative to the sub-tile's first output position; that position follows from rowptr_next
//     at the start of the range and simply advances by what each sub-tile wrote.
// Lane l owns entries l, l + 64, ... of the sub-tile, so loads and stores coalesce; the column
// indices of the next sub-tile are fetched while this one is placed.
// VALUES: every stored entry carries a value, which travels with its column index (same position); added
// entries bring theirs.  UPDATES (with VALUES): a third list, sorted like the other two, names surviving entries
// that get a new value; it is consumed through a cursor of its own, each entry finds its old entry in the staged
// columns as a deleted entry does and leaves the new value there.  An entry that names nothing stored is passed over.
template <bool VALUES, bool UPDATES>
__global__ __launch_bounds__(kWave) void merge_kernel(
    int n, const int32_t *__restrict__ rowptr_prev, const int32_t *__restrict__ colidx_prev, int nnz_prev, int range_len,
    const int32_t *__restrict__ add_row, const int32_t *__restrict__ add_col, int n_add,
    const int32_t *__restrict__ del_row, const int32_t *__restrict__ del_col, int n_del,
    const RangeStart *__restrict__ range_start,
    int32_t *__restrict__ colidx_next, int cap_next,
    const float *__restrict__ val_prev, const float *__restrict__ add_val, float *__restrict__ val_next,
    const int32_t *__restrict__ upd_row, const int32_t *__restrict__ upd_col, const float *__restrict__ upd_val, int n_upd) {
    constexpr int kWindow = 2 * kWave + 1;  // row pointers fetched ahead for every sub-tile; more are fetched when rows are short
    constexpr int kMaxWindow = kSub + kWave;
    __shared__ int s_col[kSub];
    __shared__ int s_mark[kSub + kWave];    // bit 0: deleted; bit 1: new value in s_newval; bits 2..: added entries that go right before this slot
    // Until the prefix sums are taken: s_rows[k] = rowptr_prev[first_row + k], the rows that meet the sub-tile.
    // From then on: s_start[p] = outputs (kept + added) that precede slot p's block.
    __shared__ int s_shared[kMaxWindow];
    __shared__ float s_newval[UPDATES ? kSub : 1];
    int *const s_rows = s_shared;
    int *const s_start = s_shared;
    static_assert(kMaxWindow >= kWindow + kWave, "the window must be able to grow");

    const int lane = threadIdx.x;
    const int e_begin = (int)((int64_t)blockIdx.x * range_len);
    const int e_end = (int)min((int64_t)e_begin + range_len, (int64_t)nnz_prev);
    constexpr int kNone = 0x7fffffff;    // a pointer "beyond everything"

    int c_next[kPerLane];
    float v_next[VALUES ? kPerLane : 1];
#pragma unroll
    for (int j = 0; j < kPerLane; ++j) {
        const int i = e_begin + lane + j * kWave;
        c_next[j] = i < e_end ? colidx_prev[i] : 0;
        if (VALUES) v_next[j] = i < e_end ? val_prev[i] : 0.0f;
    }

    // ---- start of the range: its row, the list cursors, the first output position
    int a_cur, d_cur;   // first added / deleted entry not yet placed
    int u_cur = 0;      // first value update not yet looked at
    int base;           // output position of the next entry to be written
    int first_row;      // the row that holds the sub-tile's first entry
    // the pointers of rows first_row + lane, first_row + 64 + lane and (lane 0) first_row + 128, for the next sub-tile
    int w0 = kNone, w1 = kNone, w2 = kNone;
    auto fetch_window = [&](int row) {
        w0 = row + lane <= n ? rowptr_prev[row + lane] : kNone;
        w1 = row + kWave + lane <= n ? rowptr_prev[row + kWave + lane] : kNone;
        w2 = (lane == 0 && row + 2 * kWave <= n) ? rowptr_prev[row + 2 * kWave] : kNone;
    };
    {
        const RangeStart st = range_start[blockIdx.x];                     // the row that holds entry e_begin
        const int rp = st.rp, rp1 = st.rp1, rn = st.rn, rn1 = st.rn1, as = st.as, ae = st.ae;
        const int ds = rp + as - rn, de = rp1 + ae - rn1;
        first_row = min(max(st.row, 0), n - 1);
        fetch_window(first_row);
        a_cur = as;
        d_cur = ds;
        if (rp < e_begin) {   // the range begins inside the row: skip what earlier ranges place
            if (as >= 0 && as < ae && ae <= n_add) a_cur = lower_bound(add_col, as, ae, colidx_prev[e_begin - 1]);
            if (ds >= 0 && ds < de && de <= n_del) d_cur = lower_bound(del_col, ds, de, colidx_prev[e_begin]);
        }
        if (UPDATES) {
            u_cur = st.us;
            if (rp < e_begin && st.us >= 0 && st.us < st.ue && st.ue <= n_upd) u_cur = lower_bound(upd_col, st.us, st.ue, colidx_prev[e_begin]);
            u_cur = min(max(u_cur, 0), n_upd);
        }
        a_cur = min(max(a_cur, 0), n_add);
        d_cur = min(max(d_cur, 0), n_del);
        base = rn + (e_begin - rp) - (d_cur - ds) + (a_cur - as);
    }
    // The 64 list entries at each cursor (row, column) are held in registers ahead of use.  A sub-tile consumes only
    // some of them: the rest slide down to lane 0 and only the freed lanes load, without anyone waiting for those
    // loads before the next sub-tile needs them.  An entry that does not exist has row kNone.
    constexpr int kVmcntZero = 0x0F70;   // s_waitcnt operand: every vector memory load has returned, other counters untouched
    int pa_row = kNone, pa_col = 0, pd_row = kNone, pd_col = 0;
    auto load_entry = [&](const int32_t *__restrict__ rows, const int32_t *__restrict__ cols, int len, int j, bool want, int &r, int &c) {
        if (want && j < len) {
            r = rows[j];
            c = cols[j];
        }
    };
    // registers hold the entries from (cur - got) on; afterwards from cur on
    auto slide = [&](const int32_t *__restrict__ rows, const int32_t *__restrict__ cols, int len, int cur, int got, int &r, int &c) {
        const int src = lane + got;
        const int r2 = __shfl(r, src & (kWave - 1), kWave);
        const int c2 = __shfl(c, src & (kWave - 1), kWave);
        const bool fresh = src >= kWave;
        c = c2;
        r = fresh ? kNone : r2;
        load_entry(rows, cols, len, cur + lane, fresh, r, c);
    };
    load_entry(add_row, add_col, n_add, a_cur + lane, true, pa_row, pa_col);
    load_entry(del_row, del_col, n_del, d_cur + lane, true, pd_row, pd_col);
    // ... and the same for the value updates, each with its value
    int pu_row = kNone, pu_col = 0;
    float pu_val = 0.0f;
    auto load_update = [&](int j, bool want) {
        if (want && j < n_upd) {
            pu_row = upd_row[j];
            pu_col = upd_col[j];
            pu_val = upd_val[j];
        }
    };
    if (UPDATES) load_update(u_cur + lane, true);

    for (int e = e_begin; e < e_end; e += kSub) {
        const int e_stop = min(e + kSub, e_end);
        const int cnt = e_stop - e;
        int c_[kPerLane];
        float v_[VALUES ? kPerLane : 1];
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) {
            c_[j] = c_next[j];
            if (VALUES) v_[j] = v_next[j];
            s_col[lane + j * kWave] = c_[j];
            s_mark[lane + j * kWave] = 0;
        }
        s_mark[kSub + lane] = 0;
        // ---- the rows that meet the sub-tile: their pointers go to LDS; `below` counts the staged pointers that are
        // <= e_stop, so the row that holds entry e_stop (the next sub-tile's first) is first_row + below - 1
        s_rows[lane] = w0;
        s_rows[kWave + lane] = w1;
        if (lane == 0) s_rows[2 * kWave] = w2;
        int n_win = kWindow;
        int last = __shfl(w2, 0, kWave);
        int below = __popcll(__ballot(w0 <= e_stop)) + __popcll(__ballot(w1 <= e_stop)) + (last <= e_stop ? 1 : 0);
#pragma unroll 1
        while (last < e_stop && n_win + kWave <= kMaxWindow) {      // short rows: the sub-tile reaches beyond the window
            const int idx = first_row + n_win + lane;
            const int v = idx <= n ? rowptr_prev[idx] : kNone;
            s_rows[n_win + lane] = v;
            below += __popcll(__ballot(v <= e_stop));
            last = __shfl(v, kWave - 1, kWave);
            n_win += kWave;
        }
        const int row0 = first_row;                  // the window staged now starts here
        first_row = min(first_row + max(below, 1) - 1, n - 1);
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) {      // fetched while this sub-tile is placed
            const int i = e_stop + lane + j * kWave;
            c_next[j] = i < e_end ? colidx_prev[i] : 0;
            if (VALUES) v_next[j] = i < e_end ? val_prev[i] : 0.0f;
        }
        if (e_stop < e_end) fetch_window(first_row);
        // the values of the (at most 64) added entries placed first in this sub-tile, fetched ahead of their use
        float av_first = 0.0f;
        if (VALUES && n_add > 0) av_first = add_val[min(a_cur + lane, n_add - 1)];
        __syncthreads();

        // where a list entry's row lies in A_prev, from the staged pointers: rows outside the window do not meet the sub-tile
        auto extent = [&](int row, int &lo, int &hi) {
            const unsigned k = (unsigned)(row - row0);
            lo = hi = kNone;
            if (k < (unsigned)(n_win - 1)) {
                lo = s_rows[k];
                hi = s_rows[k + 1];
            }
        };
        // ---- deleted entries: mark the old entry dead.  The first 64 are in registers already; a sub-tile
        // with more than that is rare and pays for its loads on the spot.
        auto strike = [&](int j) {
            bool owned = false;
            int r_lo, r_hi;
            extent(pd_row, r_lo, r_hi);
            if (j < n_del && r_lo < e_stop && r_hi > e) {      // its row has entries in this sub-tile
                const int lo = max(r_lo - e, 0), hi = min(r_hi - e, cnt);
                const int p = lds_bound<false>(s_col, lo, hi, pd_col);
                owned = p < hi && s_col[p] == pd_col;
                if (owned) atomicOr(&s_mark[p], 1);
            }
            return __popcll(__ballot(owned));
        };
        int d_got = strike(d_cur + lane);
#pragma unroll 1
        while (d_got == kWave) {
            d_cur += kWave;
            pd_row = kNone;
            load_entry(del_row, del_col, n_del, d_cur + lane, true, pd_row, pd_col);
            __builtin_amdgcn_s_waitcnt(kVmcntZero);
            d_got = strike(d_cur + lane);
        }
        d_cur += d_got;
        // ---- value updates: leave the new value at the old entry.  An entry is done with once its place in A_prev's
        // order lies before the end of this sub-tile, whether something is stored there or not.
        if (UPDATES) {
            auto touch = [&](int j) {
                bool done = false;
                int r_lo, r_hi;
                extent(pu_row, r_lo, r_hi);
                if (j < n_upd && pu_row < row0) done = true;      // a row before the sub-tile's first: nothing left to find
                else if (j < n_upd && r_lo < e_stop) {
                    const int lo = max(r_lo - e, 0), hi = min(r_hi - e, cnt);
                    const int p = lo < hi ? lds_bound<false>(s_col, lo, hi, pu_col) : hi;
                    if (p < hi) {
                        done = true;
                        if (s_col[p] == pu_col) {
                            s_newval[p] = pu_val;
                            atomicOr(&s_mark[p], 2);
                        }
                    } else {
                        done = r_hi <= e_stop;        // beyond the sub-tile's part of an unfinished row: later
                    }
                }
                return __popcll(__ballot(done));
            };
            int u_got = touch(u_cur + lane);
#pragma unroll 1
            while (u_got == kWave) {
                u_cur += kWave;
                pu_row = kNone;
                load_update(u_cur + lane, true);
                __builtin_amdgcn_s_waitcnt(kVmcntZero);
                u_got = touch(u_cur + lane);
            }
            u_cur += u_got;
            const int src = lane + u_got;       // the entries at the new cursor, for the next sub-tile
            const int r2 = __shfl(pu_row, src & (kWave - 1), kWave);
            const int c2 = __shfl(pu_col, src & (kWave - 1), kWave);
            const float v2 = __shfl(pu_val, src & (kWave - 1), kWave);
            const bool fresh = src >= kWave;
            pu_col = c2;
            pu_val = v2;
            pu_row = fresh ? kNone : r2;
            load_update(u_cur + lane, fresh);
        }
        // ---- added entries: count at the slot (old entry they precede; a row's end if none)
        const int a_tile = a_cur;
        auto slot = [&](int j, int &q) {
            bool owned = false;
            int r_lo, r_hi;
            extent(pa_row, r_lo, r_hi);
            q = -2 - lane;
            if (j < n_add && r_lo < e_stop && r_hi > e) {
                const int lo = max(r_lo - e, 0), hi = min(r_hi - e, cnt);
                q = lds_bound<true>(s_col, lo, hi, pa_col);
                owned = q < hi || r_hi <= e_stop;         // beyond the sub-tile's part of an unfinished row: later
                if (owned) atomicAdd(&s_mark[q], 4);
            }
            if (!owned) q = -2 - lane;
            return __popcll(__ballot(owned));
        };
        int q_first;                              // slot and column of the first 64, kept for the write below
        const int c_first = pa_col;
        int a_got = slot(a_cur + lane, q_first);
#pragma unroll 1
        while (a_got == kWave) {
            a_cur += kWave;
            pa_row = kNone;
            load_entry(add_row, add_col, n_add, a_cur + lane, true, pa_row, pa_col);
            __builtin_amdgcn_s_waitcnt(kVmcntZero);
            int q_unused;
            a_got = slot(a_cur + lane, q_unused);
        }
        a_cur += a_got;
        // the list entries at the new cursors, for the next sub-tile
        slide(del_row, del_col, n_del, d_cur, d_got, pd_row, pd_col);
        slide(add_row, add_col, n_add, a_cur, a_got, pa_row, pa_col);
        __syncthreads();

        // ---- prefix sums: s_start[p] = kept entries before p + added entries of slots before p (the staged row
        // pointers are not needed any more; their place is taken)
        int written;
        {
            int mk[kPerLane];
            int alive = 0, ins = 0;
#pragma unroll
            for (int j = 0; j < kPerLane; ++j) {
                const int p = lane * kPerLane + j;
                mk[j] = s_mark[p];
                alive += (p < cnt && !(mk[j] & 1)) ? 1 : 0;
                ins += mk[j] >> 2;
            }
            const int inc_alive = wave_scan_add(alive, lane), inc_ins = wave_scan_add(ins, lane);
            int run = (inc_alive - alive) + (inc_ins - ins);
#pragma unroll
            for (int j = 0; j < kPerLane; ++j) {
                const int p = lane * kPerLane + j;
                s_start[p] = run;
                run += ((p < cnt && !(mk[j] & 1)) ? 1 : 0) + (mk[j] >> 2);
            }
            if (lane == kWave - 1) s_start[kSub] = run;   // slot "after the last entry" of a full sub-tile
            written = __shfl(run, kWave - 1, kWave) + (s_mark[kSub] >> 2);
        }
        __syncthreads();

        // ---- old entries
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) {
            const int p = lane + j * kWave;
            if (p < cnt) {
                const int mk = s_mark[p];
                const unsigned pos = (unsigned)(base + s_start[p] + (mk >> 2));
                if (!(mk & 1) && pos < (unsigned)cap_next) {
                    colidx_next[pos] = c_[j];
                    if (VALUES) val_next[pos] = (UPDATES && (mk & 2)) ? s_newval[p] : v_[j];
                }
            }
        }
        // ---- added entries: their slot, then the rank among the adds of the same slot (they are consecutive).
        // The first 64 kept their slot and column from the search above; more than 64 per sub-tile are rare.
        int q_carry = -1, rank_carry = 0;
        auto place = [&](int j, int q, int c, float v) {
            const int q_left = __shfl_up(q, 1, kWave);
            const bool head = lane == 0 ? q != q_carry : q != q_left;
            const unsigned long long true_heads = __ballot(head);
            const unsigned long long upto = (true_heads | 1ull) & (~0ull >> (kWave - 1 - lane));
            const int run_start = 63 - __clzll(upto);
            int rank = lane - run_start;
            if (run_start == 0 && !(true_heads & 1ull)) rank += rank_carry;   // run continues from the previous 64
            if (j < a_cur) {
                const unsigned pos = (unsigned)(base + s_start[q] + rank);
                if (pos < (unsigned)cap_next) {
                    colidx_next[pos] = c;
                    if (VALUES) val_next[pos] = v;
                }
            }
            q_carry = __shfl(q, kWave - 1, kWave);
            rank_carry = __shfl(rank, kWave - 1, kWave) + 1;
        };
        if (a_tile < a_cur) place(a_tile + lane, q_first, c_first, av_first);
#pragma unroll 1
        for (int j0 = a_tile + kWave; j0 < a_cur; j0 += kWave) {
            // these search again; the extent of an entry's row comes from the row pointers themselves, two loads that
            // depend on the entry's, which a sub-tile this full can afford
            const int j = j0 + lane;
            int q = -2 - lane, c = 0;
            float v = 0.0f;
            if (j < a_cur) {
                const int r = add_row[j];
                c = add_col[j];
                if (VALUES) v = add_val[j];
                if ((unsigned)r < (unsigned)n) {
                    const int hi = min(rowptr_prev[r + 1] - e, cnt), lo = min(max(rowptr_prev[r] - e, 0), max(hi, 0));
                    q = lds_bound<true>(s_col, lo, hi, c);
                }
            }
            place(j, q, c, v);
        }
        base += written;
        __syncthreads();           // LDS is rewritten by the next sub-tile
    }
}

// Surviving entries whose value changes, for an update list in no particular order: one thread per listed entry
// finds it in its (new) row and overwrites the value.  Entries that are not there are skipped.
__global__ __launch_bounds__(256) void update_values_kernel(int n, const int32_t *__restrict__ rowptr,
                                                            const int32_t *__restrict__ colidx,
                                                            const int32_t *__restrict__ upd_row,
                                                            const int32_t *__restrict__ upd_col,
                                                            const float *__restrict__ upd_val, int n_upd,
                                                            float *__restrict__ val) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= n_upd) return;
    const int r = upd_row[j], c = upd_col[j];
    if ((unsigned)r >= (unsigned)n) return;
    const int lo = rowptr[r], hi = rowptr[r + 1];
    const int p = lower_bound(colidx, lo, hi, c);
    if (p < hi && colidx[p] == c) val[p] = upd_val[j];
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

// One thread per row: its pointers, then its columns one after the other (rows are short on average; a hub row
// keeps one thread busy for its length, which a check that runs once per uploaded snapshot can afford).
__global__ __launch_bounds__(256) void csr_validate_kernel(int n, const int32_t *__restrict__ rowptr,
                                                           const int32_t *__restrict__ colidx, int nnz, int require_diagonal,
                                                           int32_t *status) {
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n) return;
    const int lo = rowptr[r], hi = rowptr[r + 1];
    if ((r == 0 && lo != 0) || (r == n - 1 && hi != nnz) || lo < 0 || hi < lo || hi > nnz) {
        report(status, DGNN_BAD_ROWPTR);
        return;                                             // the row's extent cannot be trusted
    }
    bool diagonal = false;
    int prev = -1;
    for (int e = lo; e < hi; ++e) {
        const int c = colidx[e];
        if (c < 0 || c >= n) { report(status, DGNN_BAD_INDEX_RANGE); return; }
        if (c <= prev) { report(status, DGNN_BAD_ROW_ORDER); return; }
        diagonal |= c == r;
        prev = c;
    }
    if (require_diagonal && !diagonal) report(status, DGNN_BAD_NO_DIAGONAL);
}

// One thread per entry of a value-update list that is declared sorted: indices in range, strictly ascending by (row, col).
__global__ __launch_bounds__(256) void validate_updates_kernel(int n, const int32_t *__restrict__ upd_row,
                                                               const int32_t *__restrict__ upd_col, int n_upd, int32_t *status) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= n_upd) return;
    const int r = upd_row[j], c = upd_col[j];
    if (r < 0 || r >= n || c < 0 || c >= n) { report(status, DGNN_BAD_INDEX_RANGE); return; }
    if (j > 0) {
        const int pr = upd_row[j - 1], pc = upd_col[j - 1];
        if (pr > r || (pr == r && pc >= c)) report(status, DGNN_BAD_DELTA_ORDER);
    }
}

__global__ __launch_bounds__(64) void reset_status_kernel(int32_t *status) { *status = 0; }

__global__ __launch_bounds__(256) void dinv_kernel(int n, const int32_t *__restrict__ rowptr, float *__restrict__ dinv) {
    int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r < n) dinv[r] = 1.0f / sqrtf((float)(rowptr[r + 1] - rowptr[r]));
}

}  // namespace

extern "C" int dgnn_csr_validate(int64_t n, const int32_t *rowptr, const int32_t *colidx, int64_t nnz, int require_diagonal,
                                 int32_t *d_status, void *stream) {
    if (!rowptr || !d_status || (nnz > 0 && !colidx)) return DGNN_ERR_NULL;
    if (n <= 0 || nnz < 0) return DGNN_ERR_SHAPE;
    if (!fits_index(n + 1) || !fits_index(nnz)) return DGNN_ERR_OVERFLOW;
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(reset_status_kernel, dim3(1), dim3(64), 0, s, d_status);     // a fill kernel: capturable
    DGNN_RETURN_IF_LAUNCH_FAILED();
    hipLaunchKernelGGL(csr_validate_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (int)n, rowptr, colidx, (int)nnz,
                       require_diagonal, d_status);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

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
    if (!fits_index(n)) return DGNN_ERR_OVERFLOW;
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
    if (!fits_index(n_add) || !fits_index(n_del)) return DGNN_ERR_OVERFLOW;
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

namespace {

// Entries per wavefront of the merge: a multiple of the sub-tile, at most kMaxRange, smaller when the input is small.
int64_t merge_range_length(int64_t nnz_prev) {
    int64_t range_len = (nnz_prev + kTargetWaves - 1) / kTargetWaves;
    range_len = (range_len + kSub - 1) / kSub * kSub;
    return std::min<int64_t>(std::max<int64_t>(range_len, kSub), kMaxRange);
}
// No call with at most nnz_prev entries has more ranges than this (a smaller snapshot gets shorter ranges, never more
// than kTargetWaves + 1 of them), so a workspace sized for the largest snapshot of a block serves every step.
int64_t max_ranges(int64_t nnz_prev) { return std::max<int64_t>(kTargetWaves + 1, (nnz_prev + kMaxRange - 1) / kMaxRange) + 1; }

}  // namespace

extern "C" int dgnn_delta_rebuild_workspace(int64_t n, int64_t nnz_prev, int64_t n_add, int64_t n_del, size_t *bytes) {
    if (!bytes) return DGNN_ERR_NULL;
    if (n <= 0 || nnz_prev < 0 || n_add < 0 || n_del < 0) return DGNN_ERR_SHAPE;
    if (!fits_index(n + 1) || !fits_index(nnz_prev + n_add)) return DGNN_ERR_OVERFLOW;
    *bytes = round_up((size_t)max_ranges(nnz_prev) * sizeof(RangeStart), 256);   // the row every range of the merge begins in
    return DGNN_OK;
}

namespace {

struct Values {
    const float *prev;
    const float *add;
    float *next;
    // value updates the merge consumes (sorted by (row, col)); n_upd = 0: none
    const int32_t *upd_row;
    const int32_t *upd_col;
    const float *upd_val;
    int64_t n_upd;
};

int rebuild(int64_t n, const int32_t *rowptr_prev, const int32_t *colidx_prev, int64_t nnz_prev,
            const int32_t *add_row, const int32_t *add_col, int64_t n_add,
            const int32_t *del_row, const int32_t *del_col, int64_t n_del,
            int32_t *rowptr_next, int32_t *colidx_next, int64_t cap_next, int64_t *nnz_next, float *dinv_next,
            const Values *vals, void *ws, size_t ws_bytes, uint32_t flags, int32_t *d_status, void *stream) {
    if (!rowptr_prev || !colidx_prev || !rowptr_next || !colidx_next || !ws) return DGNN_ERR_NULL;
    if (n_add < 0 || n_del < 0) return DGNN_ERR_SHAPE;
    if (n_add > 0 && (!add_row || !add_col)) return DGNN_ERR_NULL;
    if (n_del > 0 && (!del_row || !del_col)) return DGNN_ERR_NULL;
    if (vals && (!vals->prev || !vals->next || (n_add > 0 && !vals->add))) return DGNN_ERR_NULL;
    if (n <= 0 || nnz_prev <= 0 || (flags & ~(vals ? DGNN_VALIDATE | DGNN_UPDATES_SORTED : DGNN_VALIDATE))) return DGNN_ERR_SHAPE;
    if (!fits_index(n + 1) || !fits_index(nnz_prev + n_add)) return DGNN_ERR_OVERFLOW;
    const int64_t nnz_new = nnz_prev + n_add - n_del;
    if (nnz_new < 0) return DGNN_ERR_SHAPE;
    if (cap_next < nnz_new) return DGNN_ERR_CAPACITY;
    const int64_t n_upd = vals ? vals->n_upd : 0;
    size_t need = 0;
    int rc = dgnn_delta_rebuild_workspace(n, nnz_prev, n_add, n_del, &need);
    if (rc != DGNN_OK) return rc;
    if (ws_bytes < need) return DGNN_ERR_CAPACITY;
    if (rowptr_next == rowptr_prev || colidx_next == colidx_prev) return DGNN_ERR_ALIAS;
    if (vals && vals->next == vals->prev) return DGNN_ERR_ALIAS;
    if (nnz_next) *nnz_next = nnz_new;

    hipStream_t s = (hipStream_t)stream;
    char *wsb = static_cast<char *>(ws);
    RangeStart *range_start = reinterpret_cast<RangeStart *>(wsb);
    const int cap = (int)min(cap_next, (int64_t)2147483647LL);
    const int64_t range_len = merge_range_length(nnz_prev);
    const int n_ranges = (int)((nnz_prev + range_len - 1) / range_len);
    const int32_t *upd_row = n_upd > 0 ? vals->upd_row : nullptr;

    const dim3 row_grid((unsigned)((n + kRowTile - 1) / kRowTile));
    if (aligned16(rowptr_prev) && aligned16(rowptr_next) && aligned16(dinv_next))
        hipLaunchKernelGGL(rowptr_kernel<true>, row_grid, dim3(kRowThreads), 0, s, (int)n, rowptr_prev, add_row, (int)n_add, del_row,
                           (int)n_del, rowptr_next, dinv_next, (int)range_len, n_ranges, range_start, upd_row, (int)n_upd, d_status);
    else
        hipLaunchKernelGGL(rowptr_kernel<false>, row_grid, dim3(kRowThreads), 0, s, (int)n, rowptr_prev, add_row, (int)n_add, del_row,
                           (int)n_del, rowptr_next, dinv_next, (int)range_len, n_ranges, range_start, upd_row, (int)n_upd, d_status);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    if ((flags & DGNN_VALIDATE) && d_status) {
        int64_t work = n_add + n_del + n;
        hipLaunchKernelGGL(validate_kernel, dim3((unsigned)((work + 255) / 256)), dim3(256), 0, s,
                           (int)n, rowptr_prev, colidx_prev, add_row, add_col, (int)n_add, del_row, del_col,
                           (int)n_del, d_status);
        DGNN_RETURN_IF_LAUNCH_FAILED();
        if (n_upd > 0) {
            hipLaunchKernelGGL(validate_updates_kernel, dim3((unsigned)((n_upd + 255) / 256)), dim3(256), 0, s, (int)n, vals->upd_row,
                               vals->upd_col, (int)n_upd, d_status);
            DGNN_RETURN_IF_LAUNCH_FAILED();
        }
    }
    const dim3 grid((unsigned)n_ranges);
    if (vals && n_upd > 0)
        hipLaunchKernelGGL((merge_kernel<true, true>), grid, dim3(kWave), 0, s, (int)n, rowptr_prev, colidx_prev, (int)nnz_prev,
                           (int)range_len, add_row, add_col, (int)n_add, del_row, del_col, (int)n_del, range_start, colidx_next, cap,
                           vals->prev, vals->add, vals->next, vals->upd_row, vals->upd_col, vals->upd_val, (int)n_upd);
    else if (vals)
        hipLaunchKernelGGL((merge_kernel<true, false>), grid, dim3(kWave), 0, s, (int)n, rowptr_prev, colidx_prev, (int)nnz_prev,
                           (int)range_len, add_row, add_col, (int)n_add, del_row, del_col, (int)n_del, range_start, colidx_next, cap,
                           vals->prev, vals->add, vals->next, nullptr, nullptr, nullptr, 0);
    else
        hipLaunchKernelGGL((merge_kernel<false, false>), grid, dim3(kWave), 0, s, (int)n, rowptr_prev, colidx_prev, (int)nnz_prev,
                           (int)range_len, add_row, add_col, (int)n_add, del_row, del_col, (int)n_del, range_start, colidx_next, cap,
                           nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

}  // namespace

extern "C" int dgnn_delta_rebuild(int64_t n,
                                  const int32_t *rowptr_prev, const int32_t *colidx_prev, int64_t nnz_prev,
                                  const int32_t *add_row, const int32_t *add_col, int64_t n_add,
                                  const int32_t *del_row, const int32_t *del_col, int64_t n_del,
                                  int32_t *rowptr_next, int32_t *colidx_next, int64_t cap_next, int64_t *nnz_next,
                                  float *dinv_next,
                                  void *ws, size_t ws_bytes, uint32_t flags, int32_t *d_status, void *stream) {
    return rebuild(n, rowptr_prev, colidx_prev, nnz_prev, add_row, add_col, n_add, del_row, del_col, n_del, rowptr_next,
                   colidx_next, cap_next, nnz_next, dinv_next, nullptr, ws, ws_bytes, flags, d_status, stream);
}

extern "C" int dgnn_delta_rebuild_weighted(int64_t n,
                                           const int32_t *rowptr_prev, const int32_t *colidx_prev, const float *val_prev,
                                           int64_t nnz_prev,
                                           const int32_t *add_row, const int32_t *add_col, const float *add_val, int64_t n_add,
                                           const int32_t *del_row, const int32_t *del_col, int64_t n_del,
                                           const int32_t *upd_row, const int32_t *upd_col, const float *upd_val, int64_t n_upd,
                                           int32_t *rowptr_next, int32_t *colidx_next, float *val_next, int64_t cap_next,
                                           int64_t *nnz_next,
                                           void *ws, size_t ws_bytes, uint32_t flags, int32_t *d_status, void *stream) {
    if (n_upd < 0) return DGNN_ERR_SHAPE;
    if (n_upd > 0 && (!upd_row || !upd_col || !upd_val)) return DGNN_ERR_NULL;
    if (!fits_index(n_upd)) return DGNN_ERR_OVERFLOW;
    const bool folded = (flags & DGNN_UPDATES_SORTED) && n_upd > 0;      // the merge takes the updates itself
    const Values vals{val_prev, add_val, val_next, upd_row, upd_col, upd_val, folded ? n_upd : 0};
    const int rc = rebuild(n, rowptr_prev, colidx_prev, nnz_prev, add_row, add_col, n_add, del_row, del_col, n_del,
                           rowptr_next, colidx_next, cap_next, nnz_next, nullptr, &vals, ws, ws_bytes, flags, d_status, stream);
    if (rc != DGNN_OK || n_upd == 0 || folded) return rc;
    hipLaunchKernelGGL(update_values_kernel, dim3((unsigned)((n_upd + 255) / 256)), dim3(256), 0, (hipStream_t)stream, (int)n,
                       rowptr_next, colidx_next, upd_row, upd_col, upd_val, (int)n_upd, val_next);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}
