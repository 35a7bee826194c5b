// One step of the sliding-window sum of snapshots, Section "Smoothening the Input Graphs":
//     C = S + alpha * A_in + beta * A_out        (S_t = S_{t-1} + A_t - A_{t-l} with alpha = 1, beta = -1)
// for a weighted snapshot S and two unweighted ones, all in CSR with sorted rows, on the device: entries of
// equal (row, column) are added up, entries whose result is exactly 0 leave the structure.  It is a three-way
// merge in the order (row, column), made into work of equal size the way the other sparse kernels here are:
// split by ENTRIES of S, not by rows, so that the hub rows of a power-law graph are spread over many lanes.
//   - a wavefront owns kRange consecutive entries of S, a lane kPer consecutive ones of those, which it keeps in
//     registers (one 16-byte load each of columns and values; the lanes' loads cover the range without a gap).  A share
//     begins at a BOUNDARY: the (row, column) of its first S entry.  Every term of A_in and A_out belongs to the
//     share whose boundary is the last one not behind it, found by one lower bound in the boundary's row; rows
//     that begin between two boundaries (rows without S entries included) belong to the share in front;
//   - the A_in and A_out terms of a range are consecutive in their arrays and are staged in LDS, with the row
//     pointers of the rows the range meets (a span longer than the staging area is read in place instead);
//   - each lane merges its share, row piece after row piece.  The merge launches are bound by the rate at which
//     the SIMDs issue vector instructions (about 600 per range and launch), not by memory;
//   - the size of the result is not known beforehand, and the host never waits for it: a first launch only counts
//     (per lane), a two-level scan turns the range totals into positions and leaves the grand total on the device,
//     the second launch merges again and writes, rowptr included -- unless the total exceeds the capacity, which
//     the write launch finds out by itself and reports in a status word.  The number of stored entries ends up
//     in rowptr_c[n]; S's own count is read from its last row pointer in the same way.
//     (One launch that counts out of LDS, learns its position from the ranges in front of it through a chained
//     scan, and writes out of LDS again was measured too: 4.2 ms per step on the largest workload against 3.3 ms
//     for the two launches -- the wavefronts hold their LDS while they wait for one another.)
// The result's order is the canonical one (rows ascending, columns ascending), whatever the launch shape.
#include <hip/hip_runtime.h>

#include "common.hpp"

namespace {

using namespace dgnn;

constexpr int kPer = 4;                // entries of S per lane (a multiple of 4: a lane fetches them 16 bytes at a time)
constexpr int kRange = kPer * kWave;   // entries of S per wavefront
constexpr int kCapIn = 80 * kPer;      // staged terms of A_in per range
constexpr int kCapOut = 64 * kPer;     // staged terms of A_out per range
constexpr int kCapRows = 32 * kPer;    // staged row pointers per range and operand
constexpr int kNoCol = 0x7fffffff;     // larger than any column index the library accepts
constexpr int kXcds = 8;
constexpr int kXcdChunk = 16;          // consecutive ranges that go to the same XCD
constexpr int kScanThreads = 1024;
constexpr int kScanTile = 4 * kScanThreads;   // counts per workgroup of the first scan level

// Where a share begins.  Rows k, k+1, ... begin at or behind the boundary; cut: the boundary lies inside row k-1.
// a, o: the first terms of A_in and A_out that are not in front of the boundary.
struct Bound { int k, cut, a, o; };

// What a lane reads besides its S entries: the terms of A_in and A_out and the row pointers of the three operands,
// from the spans staged in LDS or in place.  Staged row pointers are kept as 16-bit distances from the range's first
// S entry / A_in term / A_out term, clamped to the range's own span: every use of a row pointer below clamps it to
// (a part of) that span anyway, and a range's spans are shorter than 2^16.
template <bool STAGED>
struct Terms {
    const int *s_a, *s_o;                          // LDS: terms
    const uint16_t *s_rs, *s_ra, *s_ro;            // LDS: row pointers of rows row_off, row_off + 1, ...
    const int32_t *col_a, *col_o;                  // global
    const int32_t *rp_s, *rp_a, *rp_o;             // global; rp_a / rp_o may be null: no such operand
    int s_off, a_off, o_off, row_off;              // first S entry of the range / first staged term / row
    __device__ __forceinline__ int a(int i) const { return STAGED ? s_a[i - a_off] : col_a[i]; }
    __device__ __forceinline__ int o(int i) const { return STAGED ? s_o[i - o_off] : col_o[i]; }
    __device__ __forceinline__ int rs(int r) const { return STAGED ? s_off + s_rs[r - row_off] : rp_s[r]; }
    __device__ __forceinline__ int ra(int r) const { return STAGED ? a_off + s_ra[r - row_off] : (rp_a ? rp_a[r] : 0); }
    __device__ __forceinline__ int ro(int r) const { return STAGED ? o_off + s_ro[r - row_off] : (rp_o ? rp_o[r] : 0); }
    // first position in [b, e) whose column is >= key
    __device__ __forceinline__ int a_lower(int b, int e, int key) const {
        while (b < e) { const int mid = b + ((e - b) >> 1); if (a(mid) < key) b = mid + 1; else e = mid; }
        return b;
    }
    __device__ __forceinline__ int o_lower(int b, int e, int key) const {
        while (b < e) { const int mid = b + ((e - b) >> 1); if (o(mid) < key) b = mid + 1; else e = mid; }
        return b;
    }
    // first r in [lo, hi] with rs(r) >= key (rs(hi) >= key is known)
    __device__ __forceinline__ int first_row_at_or_after(int lo, int hi, int key) const {
        while (lo < hi) { const int mid = lo + ((hi - lo) >> 1); if (rs(mid) < key) lo = mid + 1; else hi = mid; }
        return lo;
    }
};

struct Operands {
    int n, nnz_s, nnz_a, nnz_o;                      // nnz_s: what the host was told, possibly an upper bound (see stored_s)
    const int32_t *rp_s, *col_s;
    const float *val_s;
    const int32_t *rp_a, *col_a, *rp_o, *col_o;      // rp_a / rp_o may be null: no such operand
    float alpha, beta, diag;                         // diag != 0: the value every stored diagonal entry of C takes
    int64_t capacity;                                // entries colidx_c / val_c can hold
    int s_by16;                                      // col_s and val_s can be read 16 bytes at a time
};

// The number of stored entries of S is its last row pointer (S may be the result of an earlier call, whose size the
// host never saw); never more than the host's figure, which bounds the arrays.
__device__ __forceinline__ int stored_s(const Operands &P) { return min(max(P.rp_s[P.n], 0), P.nnz_s); }

__global__ void clear_status_kernel(int32_t *d_status) { *d_status = 0; }

// The boundary at S entry `pos` (0 <= pos < nnz_s, or pos = 0 when S is empty); k_lo = first row in [k_lo, k_hi] that
// begins at pos or later, found by the caller.  Terms are looked up in [a_lo, a_hi) x [o_lo, o_hi) only (the
// spans that are known to hold the boundary).
template <bool STAGED>
__device__ __forceinline__ Bound make_bound(const Terms<STAGED> &T, int pos, int k, int col_at_pos, int a_lo, int a_hi,
                                            int o_lo, int o_hi) {
    Bound b;
    b.k = k;
    b.cut = T.rs(k) > pos;                         // k <= n and rp_s[n] = nnz_s
    if (b.cut) {                                   // inside row k-1: its terms from column col_at_pos on
        b.a = T.a_lower(max(T.ra(k - 1), a_lo), min(T.ra(k), a_hi), col_at_pos);
        b.o = T.o_lower(max(T.ro(k - 1), o_lo), min(T.ro(k), o_hi), col_at_pos);
    } else {
        b.a = T.ra(k);
        b.o = T.ro(k);
    }
    return b;
}

// One lane's share: from boundary `mine` (S entry sb0) to boundary `next` (S entry sb1); own_col, own_val: the S
// entries sb0, sb0 + 1, ...  cnt counts the results;
// WRITE: `cnt` starts at the share's position in C and the results and the row pointers of the rows that begin
// in the share are stored.
template <bool WRITE, bool STAGED>
__device__ __forceinline__ int64_t merge_share(const Operands &P, const Terms<STAGED> &T, const int (&own_col)[kPer], const float (&own_val)[kPer],
                                               const Bound &mine, int sb0, const Bound &next, int sb1, int64_t cnt,
                                               int32_t *__restrict__ rowptr_out, int32_t *__restrict__ out_col,
                                               float *__restrict__ out_val) {
    // One loop over terms AND rows: a lane whose row piece is finished moves to its next row in the same trip in
    // which other lanes merge a term, so the trip count of the wavefront is that of its longest share, not the
    // sum over row positions of the longest piece.
    int r = mine.k - (mine.cut ? 1 : 0);
    if (r >= next.k) return cnt;
    int sb = max(T.rs(r), sb0), ab = max(T.ra(r), mine.a), ob = max(T.ro(r), mine.o);
    int se = min(T.rs(r + 1), sb1), ae = min(T.ra(r + 1), next.a), oe = min(T.ro(r + 1), next.o);
    if (WRITE && r >= mine.k) rowptr_out[r] = (int32_t)cnt;                // the row begins in this share
    // the S entries not yet merged, the next one in front: registers, addressed by constants only
    int sc[kPer];
    float sv[kPer];
#pragma unroll
    for (int q = 0; q < kPer; ++q) { sc[q] = own_col[q]; sv[q] = own_val[q]; }
    for (;;) {
        const int cs = sb < se ? sc[0] : kNoCol;
        const int ca = ab < ae ? T.a(ab) : kNoCol;
        const int co = ob < oe ? T.o(ob) : kNoCol;
        const int c = min(cs, min(ca, co));
        if (c == kNoCol) {
            // next row: its pieces begin where the finished ones ended (rows are consecutive in all three arrays)
            if (++r >= next.k) break;
            se = min(T.rs(r + 1), sb1); ae = min(T.ra(r + 1), next.a); oe = min(T.ro(r + 1), next.o);
            if (WRITE) rowptr_out[r] = (int32_t)cnt;
        } else {
            float v = 0.0f;
            if (cs == c) {
                v = sv[0];
                ++sb;
#pragma unroll
                for (int q = 0; q + 1 < kPer; ++q) { sc[q] = sc[q + 1]; sv[q] = sv[q + 1]; }
            }
            if (ca == c) { v += P.alpha; ++ab; }
            if (co == c) { v += P.beta; ++ob; }
            if (c == r && P.diag != 0.0f && v != 0.0f) v = P.diag;
            if (v != 0.0f) {
                if (WRITE) { out_col[cnt] = c; out_val[cnt] = v; }
                ++cnt;
            }
        }
    }
    return cnt;
}

// bounds[w] = the boundary at S entry w * kRange (w < n_ranges), bounds[n_ranges] = the end of everything.
// A wavefront finds 64 consecutive boundaries.  Their rows lie between the rows of the first and of the last one,
// which the whole wavefront looks up together (a 64-ary search each: four dependent loads); the row pointers in
// between are staged in LDS with loads that are in flight together, and every lane searches its own row there,
// instead of a chain of two dozen dependent loads from global memory per lane.
constexpr int kBoundsTile = 2048;      // row pointers of S staged per wavefront of bounds_kernel
constexpr int kBoundsBatch = 8;        // loads a lane issues before it waits

__global__ __launch_bounds__(kWave) void bounds_kernel(Operands P, Bound *__restrict__ bounds) {
    __shared__ int s_rp[kBoundsTile];
    const int lane = threadIdx.x;
    const int w0 = blockIdx.x * kWave, w = w0 + lane;
    P.nnz_s = stored_s(P);
    const int n_ranges = max(1, (P.nnz_s + kRange - 1) / kRange);   // launched for the host's figure, never fewer
    if (w0 > n_ranges) return;
    const Terms<false> G{nullptr, nullptr, nullptr, nullptr, nullptr, P.col_a, P.col_o, P.rp_s, P.rp_a, P.rp_o, 0, 0, 0, 0};
    const int w1 = min(w0 + kWave - 1, n_ranges - 1);               // the last boundary in front of the end (w0 = n_ranges: none)
    const int p0 = (int)min((int64_t)w0 * kRange, (int64_t)P.nnz_s), p1 = (int)min((int64_t)max(w1, w0) * kRange, (int64_t)P.nnz_s);
    // first row that begins at p or later = one behind the last row that begins in front of p (rp_s[n] >= p)
    const int k0 = wave_find_row(P.rp_s, P.n + 1, p0 - 1, lane) + 1;
    const int k1 = wave_find_row(P.rp_s, P.n + 1, p1 - 1, lane) + 1;
    const int rows = k1 - k0 + 1;
    const bool tiled = rows <= kBoundsTile;
    if (tiled) {
        for (int base = 0; base < rows; base += kBoundsBatch * kWave) {
            int v[kBoundsBatch];
#pragma unroll
            for (int q = 0; q < kBoundsBatch; ++q) v[q] = P.rp_s[k0 + min(base + q * kWave + lane, rows - 1)];
#pragma unroll
            for (int q = 0; q < kBoundsBatch; ++q)
                if (base + q * kWave + lane < rows) s_rp[base + q * kWave + lane] = v[q];
        }
        wave_lds_sync();
    }
    if (w > n_ranges) return;
    if (w == n_ranges) { bounds[w] = Bound{P.n, 0, P.nnz_a, P.nnz_o}; return; }
    const int pos = (int)min((int64_t)w * kRange, (int64_t)P.nnz_s);
    int k;
    if (tiled) {
        int lo = 0, hi = rows - 1;                                  // s_rp[rows - 1] = rp_s[k1] >= p1 >= pos
        while (lo < hi) { const int mid = lo + ((hi - lo) >> 1); if (s_rp[mid] < pos) lo = mid + 1; else hi = mid; }
        k = k0 + lo;
    } else {
        k = lower_bound(P.rp_s, k0, k1, pos);
    }
    bounds[w] = make_bound(G, pos, k, pos < P.nnz_s ? P.col_s[pos] : 0, 0, P.nnz_a, 0, P.nnz_o);
}

// tiles: tiles of the scan over the range totals (of as many ranges as the host's figure for S gives).
template <bool WRITE>
__global__ __launch_bounds__(kWave) void combine_kernel(Operands P, int tiles, const Bound *__restrict__ bounds,
                                                       int32_t *__restrict__ totals, const int32_t *__restrict__ tile_off,
                                                       int32_t *__restrict__ lane_counts, int32_t *__restrict__ rowptr_out,
                                                       int32_t *__restrict__ out_col, float *__restrict__ out_val,
                                                       int32_t *__restrict__ d_status) {
    __shared__ int s_a[kCapIn];
    __shared__ int s_o[kCapOut];
    __shared__ uint16_t s_rs[kCapRows], s_ra[kCapRows], s_ro[kCapRows];

    // Workgroups are dealt to the eight XCDs in turn, and each XCD has an L2 of its own: ranges are handed out in
    // chunks of kXcdChunk consecutive ones per XCD, so that the cache lines two neighbouring ranges share (the ends
    // of their spans of A_in and A_out, their row pointers) are fetched into one L2.  The grid is a multiple of
    // kXcds * kXcdChunk, within which this is a permutation.
    const int lane = threadIdx.x;
    const int slot = blockIdx.x / kXcds, xcd = blockIdx.x % kXcds;
    const int range = ((slot / kXcdChunk) * kXcds + xcd) * kXcdChunk + slot % kXcdChunk;
    P.nnz_s = stored_s(P);
    const int n_ranges = max(1, (P.nnz_s + kRange - 1) / kRange);
    if (range >= n_ranges) {                                        // beyond what S really holds: counts nothing, writes nothing
        if (!WRITE && lane == 0) totals[range] = 0;
        return;
    }
    if (WRITE) {
        // the grand total of the count pass decides, for every range alike, whether anything is written at all
        const int64_t grand = tile_off[tiles];
        if (grand > P.capacity) {
            if (range == 0 && lane == 0) {
                rowptr_out[P.n] = (int32_t)grand;                   // the size that would have been needed
                if (d_status) atomicMax(d_status, DGNN_BAD_CAPACITY);
            }
            return;
        }
    }
    const int e0 = (int)min((int64_t)range * kRange, (int64_t)P.nnz_s), e1 = (int)min((int64_t)e0 + kRange, (int64_t)P.nnz_s);
    const bool last = range == n_ranges - 1;
    // (write pass) what the count pass and the scans left for this range, fetched with everything else
    int counted = 0;
    int64_t range_begin = 0;
    if (WRITE) {
        counted = lane_counts[(int64_t)range * kWave + lane];
        range_begin = (int64_t)totals[range] + tile_off[range / kScanTile];   // both scan levels
    }
    // This lane's share of S, entries [sb0, sb1), stays in registers: the lanes' shares are consecutive, so a
    // wavefront's 16-byte loads cover the range without a gap and nothing has to change lanes.  Issued before the
    // boundaries are known, so that everything a range needs is in flight together.
    const int sb0 = min(e0 + lane * kPer, e1), sb1 = min(sb0 + kPer, e1);
    int sc[kPer];
    float sv[kPer];
    if (P.s_by16 && sb1 - sb0 == kPer) {
#pragma unroll
        for (int q = 0; q < kPer; q += 4) {
            const uintx4 c = *reinterpret_cast<const uintx4 *>(P.col_s + sb0 + q);
            sc[q] = (int)c[0]; sc[q + 1] = (int)c[1]; sc[q + 2] = (int)c[2]; sc[q + 3] = (int)c[3];
        }
        if (P.val_s) {
#pragma unroll
            for (int q = 0; q < kPer; q += 4) {
                const uintx4 v = *reinterpret_cast<const uintx4 *>(P.val_s + sb0 + q);
                sv[q] = __uint_as_float(v[0]); sv[q + 1] = __uint_as_float(v[1]); sv[q + 2] = __uint_as_float(v[2]); sv[q + 3] = __uint_as_float(v[3]);
            }
        } else {
#pragma unroll
            for (int q = 0; q < kPer; ++q) sv[q] = 1.0f;
        }
    } else {
#pragma unroll
        for (int q = 0; q < kPer; ++q) {                           // clamped: the range's tail, or operands not 16-byte aligned
            const int src = max(min(sb0 + q, P.nnz_s - 1), 0);
            sc[q] = P.nnz_s > 0 ? P.col_s[src] : 0;
            sv[q] = (P.nnz_s > 0 && P.val_s) ? P.val_s[src] : 1.0f;
        }
    }
    // the range's own boundaries (found beforehand by bounds_kernel: one chain of dependent look-ups per range,
    // which the wavefronts in flight here could not hide)
    const Terms<false> G{nullptr, nullptr, nullptr, nullptr, nullptr, P.col_a, P.col_o, P.rp_s, P.rp_a, P.rp_o, 0, 0, 0, 0};
    const Bound B0 = bounds[range], B1 = bounds[range + 1];
    // rows whose pointers the lanes read: from the row the range begins in to the first row behind it
    const int row_lo = max(B0.k - 1, 0), row_hi = B1.k;
    const bool staged = B1.a - B0.a <= kCapIn && B1.o - B0.o <= kCapOut && row_hi - row_lo + 1 <= kCapRows;
    if (staged) {
        // Fixed numbers of loads, all issued before the first is waited for: loops over the spans' actual lengths
        // would wait for every load before issuing the next (a round trip per 64 terms).  Addresses beyond a span
        // are clamped to its last element, so that the surplus loads touch no cache line of their own.
        constexpr int kInLoads = (kCapIn + kWave - 1) / kWave, kOutLoads = (kCapOut + kWave - 1) / kWave, kRowLoads = (kCapRows + kWave - 1) / kWave;
        int va[kInLoads], vo[kOutLoads], vrs[kRowLoads], vra[kRowLoads], vro[kRowLoads];
#pragma unroll
        for (int q = 0; q < kInLoads; ++q) va[q] = B1.a > B0.a ? P.col_a[min(B0.a + q * kWave + lane, B1.a - 1)] : 0;
#pragma unroll
        for (int q = 0; q < kOutLoads; ++q) vo[q] = B1.o > B0.o ? P.col_o[min(B0.o + q * kWave + lane, B1.o - 1)] : 0;
#pragma unroll
        for (int q = 0; q < kRowLoads; ++q) {
            const int r = min(row_lo + q * kWave + lane, row_hi);
            vrs[q] = P.rp_s[r];
            vra[q] = P.rp_a ? P.rp_a[r] : 0;
            vro[q] = P.rp_o ? P.rp_o[r] : 0;
        }
#pragma unroll
        for (int q = 0; q < kInLoads; ++q) if (B0.a + q * kWave + lane < B1.a) s_a[q * kWave + lane] = va[q];
#pragma unroll
        for (int q = 0; q < kOutLoads; ++q) if (B0.o + q * kWave + lane < B1.o) s_o[q * kWave + lane] = vo[q];
#pragma unroll
        for (int q = 0; q < kRowLoads; ++q)
            if (row_lo + q * kWave + lane <= row_hi) {
                s_rs[q * kWave + lane] = (uint16_t)(min(max(vrs[q], e0), e1) - e0);
                s_ra[q * kWave + lane] = (uint16_t)(min(max(vra[q], B0.a), B1.a) - B0.a);
                s_ro[q * kWave + lane] = (uint16_t)(min(max(vro[q], B0.o), B1.o) - B0.o);
            }
        wave_lds_sync();
    }

    // an empty S still gives lane 0 of the only range a share (all rows)
    const bool active = sb0 < e1 || (P.nnz_s == 0 && lane == 0);
    auto run = [&](auto T) {
        Bound mine = B1;
        if (lane == 0) mine = B0;
        else if (active)
            mine = make_bound(T, sb0, T.first_row_at_or_after(B0.k, B1.k, sb0), sc[0], B0.a, B1.a, B0.o, B1.o);
        // the next lane's boundary; the last lane with a share ends at the range's end
        Bound next;
        next.k = __shfl_down(mine.k, 1, kWave); next.cut = __shfl_down(mine.cut, 1, kWave);
        next.a = __shfl_down(mine.a, 1, kWave); next.o = __shfl_down(mine.o, 1, kWave);
        if (lane == kWave - 1 || sb1 >= e1) next = B1;
        int64_t begin = 0;
        if (WRITE) {
            const int mine_cnt = active ? counted : 0;
            const int incl = wave_scan_add(mine_cnt, lane);
            begin = range_begin + incl - mine_cnt;
            if (last && lane == kWave - 1) rowptr_out[P.n] = (int32_t)(range_begin + incl);
        }
        int64_t end = begin;
        if (active) end = merge_share<WRITE>(P, T, sc, sv, mine, sb0, next, sb1, begin, rowptr_out, out_col, out_val);
        if (!WRITE) {
            const int cnt = (int)(end - begin);
            lane_counts[(int64_t)range * kWave + lane] = cnt;
            const int incl = wave_scan_add(cnt, lane);
            if (lane == kWave - 1) totals[range] = incl;
        }
    };
    if (staged) run(Terms<true>{s_a, s_o, s_rs, s_ra, s_ro, P.col_a, P.col_o, P.rp_s, P.rp_a, P.rp_o, e0, B0.a, B0.o, row_lo});
    else run(G);
}

// First level of the scan over range totals: every workgroup turns its tile of counts into exclusive prefix sums
// within the tile and leaves the tile's total; scan_kernel then scans the tile totals, and the write launch adds a
// range's two levels together.
__global__ __launch_bounds__(kScanThreads) void scan_tiles_kernel(int m, int32_t *__restrict__ counts, int32_t *__restrict__ tile_total) {
    constexpr int kWaves = kScanThreads / kWave;
    __shared__ int s_wave[kWaves];
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int i = blockIdx.x * kScanTile + 4 * tid;
    int v[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) v[q] = i + q < m ? counts[i + q] : 0;
    const int mine = (v[0] + v[1]) + (v[2] + v[3]);
    const int incl = wave_scan_add(mine, lane);
    if (lane == kWave - 1) s_wave[wave] = incl;
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const int t = s_wave[w];
        if (w < wave) before += t;
        total += t;
    }
    int run = before + incl - mine;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (i + q < m) counts[i + q] = run;
        run += v[q];
    }
    if (tid == 0) tile_total[blockIdx.x] = total;
}

// In place: counts[0 .. m) -> their exclusive prefix sums, counts[m] = the total.  One workgroup walks tiles of
// 4096 counts (four per thread, scanned within the wavefront by lane shifts, across wavefronts through LDS); m is
// a number of tiles of ranges, about two thousand at the largest supported snapshot.
__global__ __launch_bounds__(kScanThreads) void scan_kernel(int m, int32_t *__restrict__ counts) {
    constexpr int kWaves = kScanThreads / kWave;
    __shared__ int s_wave[kWaves];
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    int carry = 0;                                                // total of the tiles done so far (same in all threads)
    for (int base = 0; base < m; base += 4 * kScanThreads) {
        const int i = base + 4 * tid;
        int v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = i + q < m ? counts[i + q] : 0;
        const int mine = (v[0] + v[1]) + (v[2] + v[3]);
        const int incl = wave_scan_add(mine, lane);
        if (lane == kWave - 1) s_wave[wave] = incl;
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const int t = s_wave[w];
            if (w < wave) before += t;
            total += t;
        }
        int run = carry + before + incl - mine;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (i + q < m) counts[i + q] = run;
            run += v[q];
        }
        carry += total;
        __syncthreads();                                          // s_wave is written again in the next tile
    }
    if (tid == 0) counts[m] = carry;
}

int64_t range_count(int64_t nnz_s) { return std::max<int64_t>(1, (nnz_s + kRange - 1) / kRange); }
// workgroups of the merge launches: the ranges, rounded up to whole rounds of chunks over the XCDs
int64_t grid_count(int64_t nnz_s) { return (int64_t)round_up((size_t)range_count(nnz_s), (size_t)(kXcds * kXcdChunk)); }

// range totals (+ the grand total), then one count per lane
size_t totals_bytes(int64_t nnz_s) { return round_up((size_t)(4 * (grid_count(nnz_s) + 1)), (size_t)256); }
size_t counts_bytes(int64_t nnz_s) { return round_up((size_t)(4 * kWave * range_count(nnz_s)), (size_t)256); }
size_t bounds_bytes(int64_t nnz_s) { return round_up(sizeof(Bound) * (size_t)(range_count(nnz_s) + 1), (size_t)256); }
int64_t tile_count(int64_t nnz_s) { return (range_count(nnz_s) + kScanTile - 1) / kScanTile; }
size_t combine_workspace(int64_t nnz_s) {
    return totals_bytes(nnz_s) + counts_bytes(nnz_s) + bounds_bytes(nnz_s) + round_up((size_t)(4 * (tile_count(nnz_s) + 1)), (size_t)256);
}

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
                                float diag_value,
                                int32_t *rowptr_c, int32_t *colidx_c, float *val_c, int64_t capacity, int32_t *d_status,
                                void *ws, size_t ws_bytes, void *stream) {
    if (!rowptr_s || !rowptr_c || !colidx_c || !val_c || !ws) return DGNN_ERR_NULL;
    if (nnz_s > 0 && !colidx_s) return DGNN_ERR_NULL;
    if ((rowptr_in && nnz_in > 0 && !colidx_in) || (rowptr_out_of && nnz_out_of > 0 && !colidx_out_of)) return DGNN_ERR_NULL;
    if (n <= 0 || nnz_s < 0 || nnz_in < 0 || nnz_out_of < 0 || capacity < 0) return DGNN_ERR_SHAPE;
    if (!rowptr_in) nnz_in = 0;
    if (!rowptr_out_of) nnz_out_of = 0;
    if (!fits_index(n + 1) || !fits_index(nnz_s + nnz_in + nnz_out_of)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(ws)) return DGNN_ERR_ALIGN;
    if (ws_bytes < combine_workspace(nnz_s)) return DGNN_ERR_CAPACITY;
    if (rowptr_c == rowptr_s || colidx_c == colidx_s || (val_s && val_c == val_s)) return DGNN_ERR_ALIAS;
    hipStream_t s = (hipStream_t)stream;
    const int ranges = (int)range_count(nnz_s);
    int32_t *totals = (int32_t *)ws;
    int32_t *lane_counts = (int32_t *)((char *)ws + totals_bytes(nnz_s));
    const Operands P{(int)n, (int)nnz_s, (int)nnz_in, (int)nnz_out_of, rowptr_s, colidx_s, val_s, rowptr_in, colidx_in,
                     rowptr_out_of, colidx_out_of, alpha, beta, diag_value, capacity,
                     aligned16(colidx_s) && (!val_s || aligned16(val_s)) ? 1 : 0};
    Bound *bounds = (Bound *)((char *)ws + totals_bytes(nnz_s) + counts_bytes(nnz_s));
    if (d_status) {
        hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, s, d_status);
        DGNN_RETURN_IF_LAUNCH_FAILED();
    }
    hipLaunchKernelGGL(bounds_kernel, dim3((unsigned)(ranges / kWave + 1)), dim3(kWave), 0, s, P, bounds);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    const int tiles = (int)tile_count(nnz_s);
    int32_t *tile_off = (int32_t *)((char *)bounds + bounds_bytes(nnz_s));
    hipLaunchKernelGGL(combine_kernel<false>, dim3((unsigned)grid_count(nnz_s)), dim3(kWave), 0, s, P, tiles, bounds, totals, nullptr,
                       lane_counts, nullptr, nullptr, nullptr, nullptr);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    hipLaunchKernelGGL(scan_tiles_kernel, dim3((unsigned)tiles), dim3(kScanThreads), 0, s, ranges, totals, tile_off);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(kScanThreads), 0, s, tiles, tile_off);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    // the write launch reads the total where the scan left it: the host neither waits for it nor sees it
    hipLaunchKernelGGL(combine_kernel<true>, dim3((unsigned)grid_count(nnz_s)), dim3(kWave), 0, s, P, tiles, bounds, totals, tile_off,
                       lane_counts, rowptr_c, colidx_c, val_c, d_status);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}
