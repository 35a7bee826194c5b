// One step of the sliding-window sum of snapshots, Section "Smoothening the Input Graphs":
//     C = S + alpha * A_in + beta * A_out        (S_t = S_{t-1} + A_t - A_{t-l} with alpha = 1, beta = -1)
// for a weighted snapshot S and two unweighted ones, all in CSR with sorted rows, on the device: entries of
// equal (row, column) are added up, entries whose result is exactly 0 leave the structure.  It is a three-way
// merge per row, made into work of equal size the way the other sparse kernels here are: split by ENTRIES of S,
// not by rows, so that the hub rows of a power-law graph are spread over many wavefronts.
//   - a wavefront owns kRange consecutive entries of S and stages them in LDS; a row cut by the range's begin
//     or end is cut at a COLUMN (the column of the S entry the range begins or ends at), so every term of
//     A_in and A_out falls into exactly one range, found by a lower bound in its row;
//   - the A_in and A_out terms of the range are consecutive in their arrays and are staged as well (a span
//     longer than the staging area is read in place instead);
//   - each lane merges whole row pieces out of LDS, one after the other; a piece with many terms is merged by
//     all lanes, each taking an equal share of its longest list and the matching column interval of the others;
//   - the size of the result is not known beforehand: a first launch only counts (per range), a single-workgroup
//     scan turns the counts into positions, the second launch merges again and writes, rowptr included.
// The result's order is the canonical one (rows ascending, columns ascending), whatever the launch shape.
#include <hip/hip_runtime.h>

#include "common.hpp"

namespace {

using namespace dgnn;

constexpr int kRange = 1024;        // entries of S per wavefront
constexpr int kCapIn = 1536;        // staged terms of A_in per range
constexpr int kCapOut = 1024;       // staged terms of A_out per range
constexpr int kCoop = 96;           // a row piece with more terms than this is merged by all lanes together
constexpr int kNoCol = 0x7fffffff;  // larger than any column index the library accepts
constexpr int kScanThreads = 1024;

// entry i of a list is c[i - off]: the list either lies in global memory (off = 0) or a span of it is staged
struct List {
    const int32_t *c;
    int off;
    __device__ __forceinline__ int at(int i) const { return c[i - off]; }
};

// first position in [b, e) whose column is >= key
__device__ __forceinline__ int list_lower_bound(const List &l, int b, int e, int key) {
    while (b < e) {
        const int mid = b + ((e - b) >> 1);
        if (l.at(mid) < key) b = mid + 1; else e = mid;
    }
    return b;
}

// Three-way merge of S[sb, se) (columns and values in LDS, index relative to e0), A[ab, ae) and O[ob, oe).
// Returns the number of results; WRITE: stores them from position pos on.
template <bool WRITE>
__device__ __forceinline__ int merge3(const int *s_col, const float *s_val, int e0, int sb, int se, const List &A, int ab,
                                      int ae, float alpha, const List &O, int ob, int oe, float beta,
                                      int32_t *__restrict__ out_col, float *__restrict__ out_val, int64_t pos) {
    int cs = sb < se ? s_col[sb - e0] : kNoCol;
    int ca = ab < ae ? A.at(ab) : kNoCol;
    int co = ob < oe ? O.at(ob) : kNoCol;
    int cnt = 0;
    for (;;) {
        const int c = min(cs, min(ca, co));
        if (c == kNoCol) break;
        float v = 0.0f;
        if (cs == c) { v = s_val[sb - e0]; ++sb; cs = sb < se ? s_col[sb - e0] : kNoCol; }
        if (ca == c) { v += alpha; ++ab; ca = ab < ae ? A.at(ab) : kNoCol; }
        if (co == c) { v += beta; ++ob; co = ob < oe ? O.at(ob) : kNoCol; }
        if (v != 0.0f) {
            if (WRITE) { out_col[pos + cnt] = c; out_val[pos + cnt] = v; }
            ++cnt;
        }
    }
    return cnt;
}

// The share of lane `lane` when 64 lanes merge one row piece together: an equal share of the longest list, and
// of the two others the terms whose columns lie between the share's first column and the next share's.
struct Share { int sb, se, ab, ae, ob, oe; };
__device__ __forceinline__ Share coop_share(const int *s_col, int e0, int sb, int se, const List &A, int ab, int ae,
                                            const List &O, int ob, int oe, int lane) {
    const int ls = se - sb, la = ae - ab, lo = oe - ob;
    const int which = (ls >= la && ls >= lo) ? 0 : (la >= lo ? 1 : 2);
    const int lb = which == 0 ? sb : which == 1 ? ab : ob, le = which == 0 ? se : which == 1 ? ae : oe;
    const int q = (le - lb + kWave - 1) / kWave;                 // >= 1: the longest list is not empty
    const int mb = min(lb + lane * q, le), me = min(mb + q, le);
    const bool active = mb < le, first = lane == 0, final = me == le;
    auto col_of = [&](int i) { return which == 0 ? s_col[i - e0] : which == 1 ? A.at(i) : O.at(i); };
    const int c_lo = (active && !first) ? col_of(mb) : 0, c_hi = (active && !final) ? col_of(me) : 0;
    const List S{s_col, e0};
    Share sh;
    auto cut = [&](const List &l, int b, int e, int &ob_, int &oe_) {
        ob_ = first ? b : list_lower_bound(l, b, e, c_lo);
        oe_ = final ? e : list_lower_bound(l, b, e, c_hi);
        if (!active) ob_ = oe_ = e;
    };
    cut(S, sb, se, sh.sb, sh.se);
    cut(A, ab, ae, sh.ab, sh.ae);
    cut(O, ob, oe, sh.ob, sh.oe);
    return sh;
}

template <bool WRITE>
__global__ __launch_bounds__(kWave) void combine_kernel(
    int n, int nnz_s, int n_ranges, const int32_t *__restrict__ rp_s, const int32_t *__restrict__ col_s,
    const float *__restrict__ val_s, const int32_t *__restrict__ rp_a, const int32_t *__restrict__ col_a, float alpha,
    const int32_t *__restrict__ rp_o, const int32_t *__restrict__ col_o, float beta, int32_t *__restrict__ totals,
    int32_t *__restrict__ rowptr_out, int32_t *__restrict__ out_col, float *__restrict__ out_val) {
    __shared__ int s_col[kRange];
    __shared__ float s_val[kRange];
    __shared__ int s_a[kCapIn];
    __shared__ int s_o[kCapOut];

    const int lane = threadIdx.x, range = blockIdx.x;
    const int e0 = (int)min((int64_t)range * kRange, (int64_t)nnz_s), e1 = (int)min((int64_t)e0 + kRange, (int64_t)nnz_s);
    const bool last = range == n_ranges - 1;
    if (nnz_s > 0)
        for (int i = lane; i < kRange; i += kWave) {               // unconditional (clamped): the loads stay in flight together
            const int src = min(e0 + i, nnz_s - 1);
            s_col[i] = col_s[src];
            s_val[i] = val_s ? val_s[src] : 1.0f;
        }
    // rows of the range: the one cut by its begin (if any), then every row that begins in [e0, e1), rows without
    // entries included; the last range also takes the rows behind the last entry of S
    const int k_lo = wave_find_row(rp_s, n, e0 - 1, lane) + 1;           // first row that begins at e0 or later
    const int k_first = (k_lo == n || rp_s[k_lo] > e0) ? k_lo - 1 : k_lo;
    const int k_end = last ? n - 1 : wave_find_row(rp_s, n, e1 - 1, lane);
    const bool cut_l = rp_s[k_first] < e0, cut_r = rp_s[k_end + 1] > e1;
    wave_lds_sync();
    // the terms of A_in and A_out that belong to the range: whole rows, except in the cut rows, where they are
    // the ones from the column of S's entry e0 on, and below the column of S's entry e1
    const int col_l = cut_l ? s_col[0] : 0, col_r = cut_r ? col_s[e1] : 0;
    auto span = [&](const int32_t *rp, const int32_t *col, int &b, int &e) {
        b = e = 0;
        if (!rp) return;
        const List g{col, 0};
        b = cut_l ? list_lower_bound(g, rp[k_first], rp[k_first + 1], col_l) : rp[k_first];
        e = cut_r ? list_lower_bound(g, rp[k_end], rp[k_end + 1], col_r) : rp[k_end + 1];
    };
    int a_begin, a_end, o_begin, o_end;
    span(rp_a, col_a, a_begin, a_end);
    span(rp_o, col_o, o_begin, o_end);
    const bool a_staged = a_end - a_begin <= kCapIn, o_staged = o_end - o_begin <= kCapOut;
    if (a_staged) for (int i = a_begin + lane; i < a_end; i += kWave) s_a[i - a_begin] = col_a[i];
    if (o_staged) for (int i = o_begin + lane; i < o_end; i += kWave) s_o[i - o_begin] = col_o[i];
    wave_lds_sync();
    const List A{a_staged ? (const int32_t *)s_a : col_a, a_staged ? a_begin : 0};
    const List O{o_staged ? (const int32_t *)s_o : col_o, o_staged ? o_begin : 0};

    const int64_t base = WRITE ? (int64_t)totals[range] : 0;      // position of the range's first result
    int run = 0;                                                  // results of the rows handled so far
    for (int row0 = k_first; row0 <= k_end; row0 += kWave) {
        const int r = row0 + lane;
        const bool valid = r <= k_end;
        const int rb = valid ? rp_s[r] : e1, re = valid ? rp_s[r + 1] : e1;
        const bool open_l = valid && rb < e0, open_r = valid && re > e1;
        const int sb = max(rb, e0), se = min(re, e1);
        int ab = 0, ae = 0, ob = 0, oe = 0;
        if (valid && rp_a) { ab = open_l ? a_begin : rp_a[r]; ae = open_r ? a_end : rp_a[r + 1]; }
        if (valid && rp_o) { ob = open_l ? o_begin : rp_o[r]; oe = open_r ? o_end : rp_o[r + 1]; }
        const bool coop = (se - sb) + (ae - ab) + (oe - ob) > kCoop;
        // results per row piece
        int cnt = 0;
        if (valid && !coop) cnt = merge3<false>(s_col, s_val, e0, sb, se, A, ab, ae, alpha, O, ob, oe, beta, nullptr, nullptr, 0);
        const uint64_t coop_mask = __ballot(coop);
        for (uint64_t todo = coop_mask; todo; todo &= todo - 1) {
            const int src = __builtin_ctzll(todo);
            const Share sh = coop_share(s_col, e0, __shfl(sb, src, kWave), __shfl(se, src, kWave), A, __shfl(ab, src, kWave),
                                        __shfl(ae, src, kWave), O, __shfl(ob, src, kWave), __shfl(oe, src, kWave), lane);
            const int mine = merge3<false>(s_col, s_val, e0, sh.sb, sh.se, A, sh.ab, sh.ae, alpha, O, sh.ob, sh.oe, beta,
                                           nullptr, nullptr, 0);
            const int total = __shfl(wave_scan_add(mine, lane), kWave - 1, kWave);
            if (lane == src) cnt = total;
        }
        const int incl = wave_scan_add(cnt, lane);
        if (WRITE) {
            const int64_t pos = base + run + incl - cnt;          // where this lane's row piece begins
            if (valid && !open_l) rowptr_out[r] = (int32_t)pos;   // the row begins in this range
            if (valid && !coop) merge3<true>(s_col, s_val, e0, sb, se, A, ab, ae, alpha, O, ob, oe, beta, out_col, out_val, pos);
            for (uint64_t todo = coop_mask; todo; todo &= todo - 1) {
                const int src = __builtin_ctzll(todo);
                const Share sh = coop_share(s_col, e0, __shfl(sb, src, kWave), __shfl(se, src, kWave), A, __shfl(ab, src, kWave),
                                            __shfl(ae, src, kWave), O, __shfl(ob, src, kWave), __shfl(oe, src, kWave), lane);
                const int mine = merge3<false>(s_col, s_val, e0, sh.sb, sh.se, A, sh.ab, sh.ae, alpha, O, sh.ob, sh.oe, beta,
                                               nullptr, nullptr, 0);
                const int before = wave_scan_add(mine, lane) - mine;
                const int64_t row_pos = __shfl((int)(pos - base), src, kWave) + base;
                merge3<true>(s_col, s_val, e0, sh.sb, sh.se, A, sh.ab, sh.ae, alpha, O, sh.ob, sh.oe, beta, out_col, out_val,
                             row_pos + before);
            }
        }
        run += __shfl(incl, kWave - 1, kWave);
    }
    if (!WRITE && lane == 0) totals[range] = run;
    if (WRITE && last && lane == 0) rowptr_out[n] = (int32_t)(base + run);
}

// In place: counts[0 .. m) -> their exclusive prefix sums, counts[m] = the total.  One workgroup; m is a number of
// ranges, a few hundred thousand at the largest supported snapshot.
__global__ __launch_bounds__(kScanThreads) void scan_kernel(int m, int32_t *__restrict__ counts) {
    __shared__ int s_part[kScanThreads];
    const int tid = threadIdx.x;
    const int per = (m + kScanThreads - 1) / kScanThreads;
    const int b = min(tid * per, m), e = min(b + per, m);
    int sum = 0;
    for (int i = b; i < e; ++i) sum += counts[i];
    s_part[tid] = sum;
    __syncthreads();
    for (int d = 1; d < kScanThreads; d <<= 1) {                  // inclusive scan of the per-thread sums
        const int add = tid >= d ? s_part[tid - d] : 0;
        __syncthreads();
        s_part[tid] += add;
        __syncthreads();
    }
    int run = s_part[tid] - sum;
    for (int i = b; i < e; ++i) {
        const int c = counts[i];
        counts[i] = run;
        run += c;
    }
    if (tid == kScanThreads - 1) counts[m] = s_part[tid];
}

int64_t range_count(int64_t nnz_s) { return std::max<int64_t>(1, (nnz_s + kRange - 1) / kRange); }

size_t combine_workspace(int64_t nnz_s) { return round_up((size_t)(4 * (range_count(nnz_s) + 1)), (size_t)256); }

}  // namespace

extern "C" int dgnn_csr_combine_workspace(int64_t nnz_s, size_t *bytes) {
    if (!bytes) return DGNN_ERR_NULL;
    if (nnz_s < 0) return DGNN_ERR_SHAPE;
    if (!fits_index(nnz_s)) return DGNN_ERR_OVERFLOW;
    *bytes = combine_workspace(nnz_s);
    return DGNN_OK;
}

extern "C" int dgnn_csr_combine(int64_t n, const int32_t *rowptr_s, const int32_t *colidx_s, const float *val_s, int64_t nnz_s,
                                const int32_t *rowptr_in, const int32_t *colidx_in, int64_t nnz_in, float alpha,
                                const int32_t *rowptr_out_of, const int32_t *colidx_out_of, int64_t nnz_out_of, float beta,
                                int32_t *rowptr_c, int32_t *colidx_c, float *val_c, int64_t capacity, int64_t *nnz_c,
                                void *ws, size_t ws_bytes, void *stream) {
    if (!rowptr_s || !rowptr_c || !colidx_c || !val_c || !nnz_c || !ws) return DGNN_ERR_NULL;
    if (nnz_s > 0 && !colidx_s) return DGNN_ERR_NULL;
    if ((rowptr_in && nnz_in > 0 && !colidx_in) || (rowptr_out_of && nnz_out_of > 0 && !colidx_out_of)) return DGNN_ERR_NULL;
    if (n <= 0 || nnz_s < 0 || nnz_in < 0 || nnz_out_of < 0 || capacity < 0) return DGNN_ERR_SHAPE;
    if (!rowptr_in) nnz_in = 0;
    if (!rowptr_out_of) nnz_out_of = 0;
    if (!fits_index(n + 1) || !fits_index(nnz_s + nnz_in + nnz_out_of)) return DGNN_ERR_OVERFLOW;
    if (ws_bytes < combine_workspace(nnz_s)) return DGNN_ERR_CAPACITY;
    if (rowptr_c == rowptr_s || colidx_c == colidx_s || (val_s && val_c == val_s)) return DGNN_ERR_ALIAS;
    hipStream_t s = (hipStream_t)stream;
    const int ranges = (int)range_count(nnz_s);
    int32_t *totals = (int32_t *)ws;
    hipLaunchKernelGGL(combine_kernel<false>, dim3((unsigned)ranges), dim3(kWave), 0, s, (int)n, (int)nnz_s, ranges, rowptr_s,
                       colidx_s, val_s, rowptr_in, colidx_in, alpha, rowptr_out_of, colidx_out_of, beta, totals, nullptr, nullptr,
                       nullptr);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(kScanThreads), 0, s, ranges, totals);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    int32_t total = 0;
    if (hipMemcpyAsync(&total, totals + ranges, sizeof(total), hipMemcpyDeviceToHost, s) != hipSuccess) return DGNN_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return DGNN_ERR_HIP;
    *nnz_c = total;
    if (total > capacity) return DGNN_ERR_CAPACITY;
    hipLaunchKernelGGL(combine_kernel<true>, dim3((unsigned)ranges), dim3(kWave), 0, s, (int)n, (int)nnz_s, ranges, rowptr_s,
                       colidx_s, val_s, rowptr_in, colidx_in, alpha, rowptr_out_of, colidx_out_of, beta, totals, rowptr_c,
                       colidx_c, val_c);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}
