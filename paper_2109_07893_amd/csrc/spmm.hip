// Sparse factor of the GCN operation, Eqn (1) and Eqn (2): Z = sigma?(A~ H) with
// A~ = D^(-1/2) (A + I) D^(-1/2).  The snapshot is unweighted, so a stored entry (u, v) weighs
// dinv[u] * dinv[v] and the kernel needs no value array:
//     Z[u] = dinv[u] * sum_{v in row u} dinv[v] * H[v].
//
// The work is a gather of whole H rows (one 16-byte piece per lane, a lane group per row of H),
// bound by how many independent row fetches are in flight, so it is split by ENTRIES, not by
// rows, and every wavefront is an independent stream:
//   - a wavefront owns a contiguous range of stored entries and walks it in sub-tiles; the row
//     that holds the range's first entry is found once (64-ary search), afterwards rows simply
//     follow on: a window of consecutive row pointers is staged in LDS and the row starts that
//     fall into the sub-tile become a bit mask (one 32-bit word per lane group);
//   - every lane group takes 32 consecutive entries, keeps eight gathers in flight while it adds
//     up the previous eight, and closes its running sum wherever the mask has a bit: a row that
//     begins and ends inside the group's 32 entries is finished and stored at once, a piece cut
//     at either end is parked in LDS;
//   - one lane group adds the parked pieces in entry order and carries a row that is still open
//     into the next sub-tile in registers; only rows cut by the range itself leave a "left" or
//     "right" carry in the workspace, which a second small kernel adds up, again in entry order;
//   - column indices and row pointers of the next sub-tile are fetched while this one is summed.
// Hub rows of power-law graphs are thereby spread over as many wavefronts as they have ranges,
// short rows share a wavefront, and every sum has a fixed order: no floating-point atomics,
// results repeat bit for bit.
#include <algorithm>
#include <type_traits>

#include "common.hpp"

namespace {

using namespace dgnn;

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kBatch = 8;            // gathers issued together by a lane group
constexpr int kPer = 32;             // entries a lane group walks per sub-tile (one mask word)
constexpr int kMaxRange = 2048;      // entries streamed by one wavefront, at most: many short-lived wavefronts stream
                                     // faster than few long-lived ones (8192: +2.5 % on the largest workloads)
constexpr int kTargetWaves = 65536;  // ranges shrink on small inputs so that about this many wavefronts exist (16384: +4 %)
constexpr int kLongestRange = 8192;  // what a caller with little room for records may stretch a range to
constexpr int kXcds = 8;             // accelerator dies of an MI355X, each with its own L2
constexpr int kXcdChunk = 16;        // consecutive ranges that go to the same XCD
constexpr int kVmcntZero = 0x0F70;   // s_waitcnt operand: all vector memory loads returned, other counters untouched

enum : int32_t { kLeft = 1, kLeftClosed = 2, kRight = 4 };
struct RangeRec { int32_t flags, row_last, pad0, pad1; };

// ---- 16-byte feature pieces: 4 fp32 or 8 bf16, accumulated in fp32 -------------------------
template <bool BF16> struct Piece;
template <> struct Piece<false> {
    static constexpr int kVals = 4;
    typedef floatx4 Raw;
    static __device__ __forceinline__ void fma(float (&acc)[4], float s, Raw v) {
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] = fmaf(s, v[e], acc[e]);
    }
    static __device__ __forceinline__ void store(void *p, const float (&acc)[4]) {
        __builtin_nontemporal_store(floatx4{acc[0], acc[1], acc[2], acc[3]}, static_cast<floatx4 *>(p));   // written once, read by a later kernel
    }
};
template <> struct Piece<true> {
    static constexpr int kVals = 8;
    typedef uintx4 Raw;
    static __device__ __forceinline__ void fma(float (&acc)[8], float s, Raw v) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc[2 * e] = fmaf(s, __uint_as_float(v[e] << 16), acc[2 * e]);
            acc[2 * e + 1] = fmaf(s, __uint_as_float(v[e] & 0xffff0000u), acc[2 * e + 1]);
        }
    }
    static __device__ __forceinline__ void store(void *p, const float (&acc)[8]) {
        uintx4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = f32_to_bf16(acc[2 * e]) | (f32_to_bf16(acc[2 * e + 1]) << 16);
        __builtin_nontemporal_store(v, static_cast<uintx4 *>(p));
    }
};

// Z[row] piece = sigma?(dinv[row] * acc)
template <bool BF16, int NV>
__device__ __forceinline__ void finish_row(char *z, int64_t row, int row_bytes, int sub, const float *dinv, int relu,
                                           const float (&acc)[NV]) {
    const float du = dinv ? dinv[row] : 1.0f;
    float out[NV];
#pragma unroll
    for (int q = 0; q < NV; ++q) {
        out[q] = acc[q] * du;
        if (relu) out[q] = fmaxf(out[q], 0.0f);
    }
    Piece<BF16>::store(z + row * row_bytes + sub * 16, out);
}

template <bool BF16, int LPR>
__device__ __forceinline__ void zero_row(char *z, int64_t row) {
    constexpr int NV = Piece<BF16>::kVals;
    float zero[NV];
#pragma unroll
    for (int q = 0; q < NV; ++q) zero[q] = 0.0f;
    for (int s = 0; s < LPR; ++s) Piece<BF16>::store(z + row * (LPR * 16) + s * 16, zero);
}

// LPR: lanes per feature row.  SCALE_V: multiply every gathered row by a per-entry factor: dinv of its
// column, or the entry's own value when the snapshot carries values (otherwise H already carries the factor).
template <int LPR, bool BF16, bool SCALE_V>
__global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(4, 8))) void spmm_stream_kernel(
    int n, int nnz, int range_len, int n_ranges, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const float *__restrict__ dinv, const char *__restrict__ h, char *__restrict__ z, int relu,
    RangeRec *__restrict__ recs, float *__restrict__ carry, const float *__restrict__ vals) {
    typedef typename Piece<BF16>::Raw Raw;
    constexpr int NV = Piece<BF16>::kVals;
    constexpr int F = LPR * NV;
    constexpr int G = kWave / LPR;          // lane groups per wavefront
    constexpr int SUB = G * kPer;           // entries per sub-tile
    constexpr int CPL = kPer / LPR;         // column indices held by one lane
    constexpr int kRowBytes = LPR * 16;
    constexpr int kRowCap = SUB + kWave;    // most rows a sub-tile can need: one per entry, plus the bounding one
    constexpr int ROUNDS = kRowCap / kWave;

    __shared__ int s_rp[kRowCap];           // row pointers of the staged rows
    __shared__ float s_du[kRowCap];         // their dinv
    __shared__ unsigned s_heads[G + 1];     // bit p of the mask: a row begins at entry e + p
    __shared__ float s_part[G][2][F];       // [0]: a group's first piece when cut on the left, [1]: its last piece when cut on the right only

    const int lane = threadIdx.x;
    const int sub = lane % LPR, g = lane / LPR, gbase = lane - sub;
    // Workgroups are dealt to the eight XCDs in turn, and each XCD has an L2 of its own.  Ranges are handed
    // out in chunks of kXcdChunk consecutive ones per XCD, so that rows which lie close together (and in a
    // graph with locality gather the same rows of H) meet in one L2, while every XCD still gets a share of
    // every part of the matrix (parts differ in cost per entry when row lengths are clustered).
    const int slot = blockIdx.x / kXcds, xcd = blockIdx.x % kXcds;
    const int range = ((slot / kXcdChunk) * kXcds + xcd) * kXcdChunk + slot % kXcdChunk;
    if (range >= n_ranges) return;
    // the host's count may be an upper bound (a snapshot whose size only the device knows): the last row pointer decides
    nnz = min(nnz, rowptr[n]);
    const int e_begin = (int)((int64_t)range * range_len);
    if (e_begin >= nnz && range > 0) {                  // nothing stored here: a record that closes nothing and carries nothing
        if (threadIdx.x == 0) recs[range] = RangeRec{0, 0, 0, 0};
        return;
    }
    const int e_end = (int)min((int64_t)e_begin + range_len, (int64_t)nnz);
    int k_cur = max(wave_find_row(rowptr, n, e_begin, lane), 0);   // a row with rowptr <= e_begin
    if (range == 0)                          // rows without entries ahead of the first stored entry
        for (int k = lane; k < k_cur; k += kWave) zero_row<BF16, LPR>(z, k);

    // the row that is still open at the end of a sub-tile is carried on in the lanes of group 0
    float run[NV];
#pragma unroll
    for (int q = 0; q < NV; ++q) run[q] = 0.0f;
    bool running = false;       // such a row exists
    bool began_here = false;    // ... and it began inside this range
    int run_row = 0;
    int range_flags = 0;
    float *my_carry = carry + (int64_t)range * 2 * F;

    // column indices (and their dinv) of the coming sub-tile: lane holds entries e + 32 g + sub CPL + i
    int c_next[CPL];
    float d_next[SCALE_V ? CPL : 1];
    auto fetch_cols = [&](int e0) {
#pragma unroll
        for (int i = 0; i < CPL; ++i) {
            const int idx = e0 + g * kPer + sub * CPL + i;
            c_next[i] = idx < e_end ? __builtin_nontemporal_load(colidx + idx) : 0;   // a stream: the caches are for rows of H
        }
        if (SCALE_V) {
#pragma unroll
            for (int i = 0; i < CPL; ++i) {
                const int idx = e0 + g * kPer + sub * CPL + i;
                // an explicit value per stored entry (one coalesced stream), else dinv of the entry's column
                d_next[i] = idx < e_end ? (vals ? vals[idx] : dinv[c_next[i]]) : 0.0f;
            }
        }
    };
    // row pointers (and dinv) of the first 64 rows of the coming sub-tile; further rows are read on demand
    int m_v = 0;
    float m_du = 1.0f;
    auto fetch_rows = [&](int k0) {
        const int k = k0 + lane;
        m_v = k <= n ? rowptr[k] : 0x7fffffff;
        m_du = (dinv && k < n) ? dinv[k] : 1.0f;
    };
    fetch_cols(e_begin);
    fetch_rows(k_cur);
    int k_win = k_cur, staged_last = kWave;   // the last staged window, for the rows beyond it
    int e = e_begin;
    while (e < e_end) {
        // ---- stage rows k_cur, k_cur + 1, ... in LDS until one begins at or beyond the end of the sub-tile
        const int e_lim = min(e + SUB, e_end);
        int staged = 0, le_e = 0, le_stop = 0, lt_stop = 0;
        bool complete = false;
        {
            int v = m_v;
            float du = m_du;
#pragma unroll 1
            for (int round = 0; round < ROUNDS && !complete; ++round) {
                const int t = lane + round * kWave;
                if (round > 0) {
                    const int k = k_cur + t;
                    v = k <= n ? rowptr[k] : 0x7fffffff;
                    du = (dinv && k < n) ? dinv[k] : 1.0f;
                }
                s_rp[t] = v;
                s_du[t] = du;
                le_e += __popcll(__ballot(v <= e));
                le_stop += __popcll(__ballot(v <= e_lim));
                lt_stop += __popcll(__ballot(v < e_lim));
                staged += kWave;
                complete = __ballot(v >= e_lim) != 0;
            }
        }
        k_win = k_cur;
        staged_last = staged;
        const int t0 = max(le_e - 1, 0);                 // the staged row that holds entry e
        __syncthreads();
        // rows without entries give zero output (none exist when every row holds its diagonal)
#pragma unroll 1
        for (int t = lane; t + 1 < staged; t += kWave)
            if (k_cur + t + 1 <= n && s_rp[t] == s_rp[t + 1]) zero_row<BF16, LPR>(z, k_cur + t);
        if (t0 > 0) {                                    // rows without entries were stepped over: restage from the row of e
            k_cur += t0;
            fetch_rows(k_cur);
            __syncthreads();
            continue;
        }
        int e_stop = e_lim;
        if (!complete) {                                 // more rows begin here than fit (rows without entries): end early
            e_stop = min(e_lim, s_rp[staged - 1]);
            le_stop = lt_stop = 0;
#pragma unroll 1
            for (int t = lane; t - lane < staged; t += kWave) {
                const int v = t < staged ? s_rp[t] : 0x7fffffff;
                le_stop += __popcll(__ballot(v <= e_stop));
                lt_stop += __popcll(__ballot(v < e_stop));
            }
        }
        const int cnt = e_stop - e;
        const int t_last = lt_stop - 1;                  // last staged row with entries in this sub-tile
        const int k_next = k_cur + le_stop - 1;          // a row with rowptr <= e_stop

        int cc[CPL];
        float dd[SCALE_V ? CPL : 1];
#pragma unroll
        for (int i = 0; i < CPL; ++i) {
            cc[i] = c_next[i];
            if (SCALE_V) dd[i] = d_next[i];
        }
        if (lane <= G) s_heads[lane] = 0u;
        // Every load issued so far has been used or is used next; saying so here, ahead of the prefetch, keeps
        // the gathers below from being held up by waits for "possibly outstanding" column indices.
        __builtin_amdgcn_s_waitcnt(kVmcntZero);
        if (e_stop < e_end) {                            // fetched while this sub-tile is summed
            fetch_cols(e_stop);
            fetch_rows(k_next);
        }
        __syncthreads();
        // ---- row starts inside the sub-tile -> mask bits
#pragma unroll 1
        for (int t = lane; t < staged; t += kWave) {
            const int v = s_rp[t];
            if (t > 0 && v < e_stop) {
                const int p = v - e;
                atomicOr(&s_heads[p >> 5], 1u << (p & 31));
            }
        }
        if (lane == 0 && s_rp[0] == e) atomicOr(&s_heads[0], 1u);
        __syncthreads();

        // ---- every lane group walks its 32 entries
        const int p0 = g * kPer;
        const int c1 = min(p0 + kPer, cnt);
        if (p0 < c1) {
            const unsigned w = s_heads[g];
            int cur;                                     // staged row that holds entry p0: last one that begins at or before it
            {
                int lo = 0, hi = t_last + 1;
                while (lo < hi) {
                    const int mid = lo + ((hi - lo) >> 1);
                    if (s_rp[mid] <= e + p0) lo = mid + 1; else hi = mid;
                }
                cur = lo - 1;
            }
            bool left_closed = (w & 1u) != 0;            // entry p0 begins its row
            float acc[NV];
#pragma unroll
            for (int q = 0; q < NV; ++q) acc[q] = 0.0f;

            // a piece that is a whole row is finished and stored; a cut piece is parked for the step below
            auto flush = [&](bool right_closed) {
                if (left_closed && right_closed) {
                    float out[NV];
                    const float du = s_du[cur];
#pragma unroll
                    for (int q = 0; q < NV; ++q) {
                        out[q] = acc[q] * du;
                        if (relu) out[q] = fmaxf(out[q], 0.0f);
                    }
                    Piece<BF16>::store(z + (int64_t)(k_cur + cur) * kRowBytes + sub * 16, out);
                } else {
                    float *dst = &s_part[g][left_closed ? 1 : 0][sub * NV];
#pragma unroll
                    for (int q = 0; q < NV; ++q) dst[q] = acc[q];
                }
            };
            // batch b covers entries 8 b .. 8 b + 7 of the group; ODD (the parity of b) makes the register
            // slot q % CPL a compile-time constant while b itself stays a run-time loop counter
            // FULL: all 32 entries of every group exist (any sub-tile but a range's last), so nothing about the
            // gathers is conditional and each one is waited for by itself, in the order they were issued
            auto batch = [&](int b, auto odd, auto full) {
                constexpr int ODD = decltype(odd)::value;
                constexpr bool FULL = decltype(full)::value;
                constexpr int slot_odd = (ODD * kBatch) % CPL;
                Raw buf[kBatch];
#pragma unroll
                for (int k = 0; k < kBatch; ++k) {
                    const int q = b * kBatch + k;
                    if (FULL || p0 + q < c1) {
                        const int c = __shfl(cc[(slot_odd + k) % CPL], gbase + q / CPL, kWave);
                        buf[k] = *reinterpret_cast<const Raw *>(h + (int64_t)c * kRowBytes + sub * 16);
                    }
                }
                const unsigned wb = w >> (b * kBatch);
#pragma unroll
                for (int k = 0; k < kBatch; ++k) {
                    const int q = b * kBatch + k;
                    if (FULL || p0 + q < c1) {
                        if (q > 0 && ((wb >> k) & 1u)) {
                            flush(true);
                            left_closed = true;
                            do ++cur; while (s_rp[cur + 1] <= e + p0 + q);   // rows without entries are stepped over
#pragma unroll
                            for (int x = 0; x < NV; ++x) acc[x] = 0.0f;
                        }
                        const float s = SCALE_V ? __shfl(dd[(slot_odd + k) % CPL], gbase + q / CPL, kWave) : 1.0f;
                        Piece<BF16>::fma(acc, s, buf[k]);
                    }
                }
            };
            if (cnt == SUB) {
#pragma unroll 1
                for (int b = 0; b < kPer / kBatch; b += 2) {
                    batch(b, std::integral_constant<int, 0>{}, std::true_type{});
                    batch(b + 1, std::integral_constant<int, 1>{}, std::true_type{});
                }
            } else {
#pragma unroll 1
                for (int b = 0; b < kPer / kBatch; b += 2) {
                    batch(b, std::integral_constant<int, 0>{}, std::false_type{});
                    batch(b + 1, std::integral_constant<int, 1>{}, std::false_type{});
                }
            }
            // does the row of the last entry end with it?
            flush(c1 == cnt ? s_rp[t_last + 1] == e_stop : (s_heads[g + 1] & 1u) != 0);
        }
        __syncthreads();

        // ---- rows cut between lane groups or by the sub-tile: their pieces are added in entry order.
        // Where a row's pieces lie follows from the row pointers alone.
        auto pieces = [&](int t, float (&sum)[NV]) {
            const int ps = s_rp[t] - e;
            const int pe = min(s_rp[t + 1] - e, cnt);
            const int ga = max(ps, 0) >> 5, gb = (pe - 1) >> 5;
            int first = ga;
#pragma unroll
            for (int q = 0; q < NV; ++q) sum[q] = 0.0f;
            if (ps >= 0) {                               // begins here: its first piece is the last one of group ga
#pragma unroll
                for (int q = 0; q < NV; ++q) sum[q] = s_part[ga][1][sub * NV + q];
                first = ga + 1;
            }
            for (int gg = first; gg <= gb; ++gg)
#pragma unroll
                for (int q = 0; q < NV; ++q) sum[q] += s_part[gg][0][sub * NV + q];
        };
        for (int t = 1 + g; t < t_last; t += G) {        // rows strictly inside the sub-tile
            const int ps = s_rp[t] - e, pe = s_rp[t + 1] - e;
            if (pe > ps && (ps >> 5) != ((pe - 1) >> 5)) {
                float sum[NV];
                pieces(t, sum);
                float out[NV];
#pragma unroll
                for (int q = 0; q < NV; ++q) {
                    out[q] = sum[q] * s_du[t];
                    if (relu) out[q] = fmaxf(out[q], 0.0f);
                }
                Piece<BF16>::store(z + (int64_t)(k_cur + t) * kRowBytes + sub * 16, out);
            }
        }
        if (lane < LPR) {                                // the first and the last row of the sub-tile
            const bool first_starts = s_rp[0] == e, first_ends = s_rp[1] <= e_stop;
            const bool first_whole_in_group = first_starts && first_ends && ((s_rp[1] - e - 1) >> 5) == 0;
            if (!first_whole_in_group) {
                float sum[NV];
                pieces(0, sum);
                if (first_starts) {                      // nothing is being carried: this row begins the carry
#pragma unroll
                    for (int q = 0; q < NV; ++q) run[q] = sum[q];
                    running = true;
                    began_here = true;
                    run_row = k_cur;
                } else {
#pragma unroll
                    for (int q = 0; q < NV; ++q) run[q] += sum[q];
                    if (!running) { running = true; began_here = false; run_row = k_cur; }
                }
                if (first_ends) {
                    if (began_here) {
                        finish_row<BF16, NV>(z, (int64_t)run_row, kRowBytes, lane, dinv, relu, run);
                    } else {                             // end of the row inherited from the previous range
#pragma unroll
                        for (int q = 0; q < NV; ++q) my_carry[lane * NV + q] = run[q];
                        range_flags |= kLeft | kLeftClosed;
                    }
                    running = false;
#pragma unroll
                    for (int q = 0; q < NV; ++q) run[q] = 0.0f;
                }
            }
            if (t_last > 0) {
                const bool last_ends = s_rp[t_last + 1] <= e_stop;
                const int ps = s_rp[t_last] - e;
                const bool last_whole_in_group = last_ends && (ps >> 5) == ((e_stop - e - 1) >> 5);
                if (!last_whole_in_group) {
                    float sum[NV];
                    pieces(t_last, sum);
                    if (last_ends) {
                        float out[NV];
#pragma unroll
                        for (int q = 0; q < NV; ++q) {
                            out[q] = sum[q] * s_du[t_last];
                            if (relu) out[q] = fmaxf(out[q], 0.0f);
                        }
                        Piece<BF16>::store(z + (int64_t)(k_cur + t_last) * kRowBytes + lane * 16, out);
                    } else {                             // goes on in the next sub-tile
#pragma unroll
                        for (int q = 0; q < NV; ++q) run[q] = sum[q];
                        running = true;
                        began_here = true;
                        run_row = k_cur + t_last;
                    }
                }
            }
        }
        k_cur = k_next;
        e = e_stop;
        __syncthreads();
    }

    if (lane < LPR) {
        if (running) {
            if (began_here) {                            // goes on in the next range
#pragma unroll
                for (int q = 0; q < NV; ++q) my_carry[F + lane * NV + q] = run[q];
                range_flags |= kRight;
            } else {                                     // the whole range lies inside one row
#pragma unroll
                for (int q = 0; q < NV; ++q) my_carry[lane * NV + q] = run[q];
                range_flags |= kLeft;
            }
        }
        if (lane == 0) recs[range] = RangeRec{range_flags, run_row, 0, 0};
    }
    if (e_end == nnz)                                    // rows without entries beyond the last staged window
        for (int k = k_win + staged_last - 1 + lane; k < n; k += kWave)
            if (rowptr[k] == rowptr[k + 1]) zero_row<BF16, LPR>(z, k);
}

// Rows cut by range boundaries: the range where such a row begins owns it and adds the left carries
// of the following ranges until the one that closes the row.
template <int LPR, bool BF16>
__global__ __launch_bounds__(256) void spmm_carry_kernel(int ranges, const RangeRec *__restrict__ recs,
                                                         const float *__restrict__ carry,
                                                         const float *__restrict__ dinv, char *__restrict__ z, int relu) {
    constexpr int NV = Piece<BF16>::kVals;
    constexpr int F = LPR * NV;
    constexpr int G = 256 / LPR;
    const int tid = threadIdx.x;
    const int sub = tid % LPR;
    const int t = blockIdx.x * G + tid / LPR;
    if (t >= ranges) return;
    const RangeRec rec = recs[t];
    if (!(rec.flags & kRight)) return;
    float acc[NV];
#pragma unroll
    for (int q = 0; q < NV; ++q) acc[q] = carry[((int64_t)t * 2 + 1) * F + sub * NV + q];
    for (int j = t + 1; j < ranges; ++j) {
        const int fj = recs[j].flags;
        if (!(fj & kLeft)) break;
#pragma unroll
        for (int q = 0; q < NV; ++q) acc[q] += carry[(int64_t)j * 2 * F + sub * NV + q];
        if (fj & kLeftClosed) break;
    }
    finish_row<BF16, NV>(z, (int64_t)rec.row_last, LPR * 16, sub, dinv, relu, acc);
}

struct Workspace {
    RangeRec *recs;
    float *carry;
};

// Entries per wavefront: a multiple of the sub-tile, at most kMaxRange, smaller when the input is small.
// max_ranges > 0: the caller has room for that many range records only; ranges are stretched to fit, up to
// kLongestRange (0 is returned if even that does not do).
int range_length(int64_t nnz, int sub_tile, int64_t max_ranges = 0) {
    int64_t len = (nnz + kTargetWaves - 1) / kTargetWaves;
    len = (len + sub_tile - 1) / sub_tile * sub_tile;
    if (len > kMaxRange) len = kMaxRange;
    if (max_ranges > 0 && (nnz + len - 1) / len > max_ranges) {
        len = (nnz + max_ranges - 1) / max_ranges;
        len = (len + sub_tile - 1) / sub_tile * sub_tile;
        if (len > kLongestRange) return 0;
    }
    return (int)len;
}

// Sized for the largest number of ranges any call with at most nnz entries can have (a smaller snapshot gets
// shorter ranges, never more than kTargetWaves + 1 of them), so a buffer queried for the largest snapshot of a
// block serves every snapshot of it, and both dtypes.
size_t workspace_layout(int64_t nnz, int32_t f, Workspace *ws, void *base, int64_t exact_ranges = 0) {
    // exact_ranges: the number of ranges of one particular call (a caller that knows the call and has little room)
    const int64_t ranges = exact_ranges > 0 ? exact_ranges
                                            : std::max<int64_t>(kTargetWaves + 1, (nnz + kMaxRange - 1) / kMaxRange) + 1;
    const size_t o_carry = round_up((size_t)ranges * sizeof(RangeRec), 256);
    const size_t total = o_carry + round_up((size_t)ranges * 2 * f * sizeof(float), 256);
    if (ws) {
        char *b = static_cast<char *>(base);
        ws->recs = reinterpret_cast<RangeRec *>(b);
        ws->carry = reinterpret_cast<float *>(b + o_carry);
    }
    return total;
}

template <int LPR, bool BF16>
int launch(int64_t n, int64_t nnz, int range_len, const int32_t *rowptr, const int32_t *colidx, const float *dinv, bool scale_v,
           const void *h, void *z, int relu, const Workspace &ws, hipStream_t s, const float *vals = nullptr) {
    constexpr int G = 256 / LPR;
    const int ranges = (int)((nnz + range_len - 1) / range_len);
    const int grid = (ranges + kXcds * kXcdChunk - 1) / (kXcds * kXcdChunk) * (kXcds * kXcdChunk);   // whole chunk rounds
    if (scale_v)
        hipLaunchKernelGGL((spmm_stream_kernel<LPR, BF16, true>), dim3(grid), dim3(kWave), 0, s, (int)n, (int)nnz, range_len, ranges,
                           rowptr, colidx, dinv, static_cast<const char *>(h), static_cast<char *>(z), relu, ws.recs, ws.carry, vals);
    else
        hipLaunchKernelGGL((spmm_stream_kernel<LPR, BF16, false>), dim3(grid), dim3(kWave), 0, s, (int)n, (int)nnz, range_len, ranges,
                           rowptr, colidx, dinv, static_cast<const char *>(h), static_cast<char *>(z), relu, ws.recs, ws.carry, vals);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    hipLaunchKernelGGL((spmm_carry_kernel<LPR, BF16>), dim3((ranges + G - 1) / G), dim3(256), 0, s, ranges, ws.recs,
                       ws.carry, dinv, static_cast<char *>(z), relu);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

}  // namespace

extern "C" int dgnn_spmm_workspace(int64_t n, int64_t nnz, int32_t f, size_t *bytes) {
    if (!bytes) return DGNN_ERR_NULL;
    if (n <= 0 || nnz < 0 || !supported_width(f)) return DGNN_ERR_SHAPE;
    if (!fits_index(n + 1) || !fits_index(nnz)) return DGNN_ERR_OVERFLOW;
    *bytes = workspace_layout(nnz, f, nullptr, nullptr);
    return DGNN_OK;
}

namespace {

// Entries per range of one call for this snapshot, width and storage type (max_ranges as in range_length).
int range_length_of_call(int64_t nnz, int32_t f, dgnn_dtype dt, int64_t max_ranges = 0) {
    const int lpr = dt == DGNN_F32 ? f / 4 : f / 8;
    return range_length(nnz, (kWave / lpr) * kPer, max_ranges);
}

int spmm(int64_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *dinv, const float *vals,
         const void *h, int32_t f, void *z, dgnn_dtype dt, uint32_t flags, uint32_t allowed, void *ws, size_t ws_bytes,
         void *stream, int64_t max_ranges = 0) {
    if (!rowptr || !colidx || !h || !z || !ws) return DGNN_ERR_NULL;
    if (n <= 0 || nnz <= 0 || !supported_width(f) || (flags & ~allowed)) return DGNN_ERR_SHAPE;
    if (dt != DGNN_F32 && dt != DGNN_BF16) return DGNN_ERR_SHAPE;
    if (!fits_index(n + 1) || !fits_index(nnz)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(h) || !aligned16(z) || !aligned16(ws)) return DGNN_ERR_ALIGN;
    if (h == z) return DGNN_ERR_ALIAS;
    // max_ranges > 0: the records of exactly this call, laid out for its own number of ranges
    const int range_len = range_length_of_call(nnz, f, dt, max_ranges);
    if (range_len <= 0) return DGNN_ERR_CAPACITY;
    Workspace w;
    if (ws_bytes < workspace_layout(nnz, f, &w, ws, max_ranges > 0 ? (nnz + range_len - 1) / range_len : 0)) return DGNN_ERR_CAPACITY;
    hipStream_t s = (hipStream_t)stream;
    const int relu = (flags & DGNN_RELU) ? 1 : 0;
    const bool scale_v = vals != nullptr || (dinv != nullptr && !(flags & DGNN_H_PRESCALED));
    const int lpr = dt == DGNN_F32 ? f / 4 : f / 8;   // lanes per feature row, 16 bytes each
    const bool bf = dt == DGNN_BF16;
    switch (lpr) {
        case 2: return launch<2, true>(n, nnz, range_len, rowptr, colidx, dinv, scale_v, h, z, relu, w, s, vals);
        case 4: return bf ? launch<4, true>(n, nnz, range_len, rowptr, colidx, dinv, scale_v, h, z, relu, w, s, vals)
                          : launch<4, false>(n, nnz, range_len, rowptr, colidx, dinv, scale_v, h, z, relu, w, s, vals);
        case 8: return bf ? launch<8, true>(n, nnz, range_len, rowptr, colidx, dinv, scale_v, h, z, relu, w, s, vals)
                          : launch<8, false>(n, nnz, range_len, rowptr, colidx, dinv, scale_v, h, z, relu, w, s, vals);
        case 16: return bf ? launch<16, true>(n, nnz, range_len, rowptr, colidx, dinv, scale_v, h, z, relu, w, s, vals)
                           : launch<16, false>(n, nnz, range_len, rowptr, colidx, dinv, scale_v, h, z, relu, w, s, vals);
        case 32: return launch<32, false>(n, nnz, range_len, rowptr, colidx, dinv, scale_v, h, z, relu, w, s, vals);
        default: return DGNN_ERR_SHAPE;
    }
}

}  // namespace

extern "C" int dgnn_spmm(int64_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *dinv,
                         const void *h, int32_t f, void *z, dgnn_dtype dt, uint32_t flags,
                         void *ws, size_t ws_bytes, void *stream) {
    return spmm(n, nnz, rowptr, colidx, dinv, nullptr, h, f, z, dt, flags, DGNN_RELU | DGNN_H_PRESCALED, ws, ws_bytes, stream);
}

// ---- the same aggregation for callers that cannot allocate: its carry records live in a file-scope device array ----
namespace {

constexpr size_t kStaticScratchBytes = size_t(32) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void *g_scratch_ptr[kMaxDevices];   // per device: the address of that device's copy of `scratch`, asked for once

// The device address of the current device's `scratch` (the array's name is only a host-side handle).
int static_scratch(void **out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return DGNN_ERR_HIP;
    }
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return DGNN_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DGNN_OK;
}

}  // namespace

extern "C" int dgnn_spmm_static_limit(size_t *bytes) {
    if (!bytes) return DGNN_ERR_NULL;
    *bytes = kStaticScratchBytes;
    return DGNN_OK;
}

extern "C" int dgnn_spmm_static(int64_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *dinv,
                                const void *h, int32_t f, void *z, dgnn_dtype dt, uint32_t flags, void *stream) {
    // argument errors first, so that they are reported without touching the device
    if (!rowptr || !colidx || !h || !z) return DGNN_ERR_NULL;
    if (n <= 0 || nnz <= 0 || !supported_width(f) || (flags & ~(DGNN_RELU | DGNN_H_PRESCALED))) return DGNN_ERR_SHAPE;
    if (dt != DGNN_F32 && dt != DGNN_BF16) return DGNN_ERR_SHAPE;
    if (!fits_index(n + 1) || !fits_index(nnz)) return DGNN_ERR_OVERFLOW;
    // as many ranges as the array has room for records of: ranges grow longer where the usual ones would be too many
    const int64_t max_ranges = (int64_t)((kStaticScratchBytes - 512) / (sizeof(RangeRec) + 2 * (size_t)f * sizeof(float)));
    if (range_length_of_call(nnz, f, dt, max_ranges) <= 0) return DGNN_ERR_CAPACITY;
    void *ptr = nullptr;
    const int rc = static_scratch(&ptr);
    if (rc != DGNN_OK) return rc;
    // every range writes its record and the carries its flags announce before the second kernel reads them, so nothing
    // in the array has to start at zero; what the previous call left there is never read
    return spmm(n, nnz, rowptr, colidx, dinv, nullptr, h, f, z, dt, flags, DGNN_RELU | DGNN_H_PRESCALED, ptr,
                kStaticScratchBytes, stream, max_ranges);
}

extern "C" int dgnn_spmm_weighted(int64_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *val,
                                  const float *dinv, const void *h, int32_t f, void *z, dgnn_dtype dt, uint32_t flags,
                                  void *ws, size_t ws_bytes, void *stream) {
    if (!val) return DGNN_ERR_NULL;
    // with a normalisation the right-hand factor must already be in the rows of h: the kernel gathers one
    // per-entry factor (the value), not two
    if (dinv && !(flags & DGNN_H_PRESCALED)) return DGNN_ERR_SHAPE;
    if (!dinv && (flags & DGNN_H_PRESCALED)) return DGNN_ERR_SHAPE;
    return spmm(n, nnz, rowptr, colidx, dinv, val, h, f, z, dt, flags, DGNN_RELU | DGNN_H_PRESCALED, ws, ws_bytes, stream);
}

namespace {

// ---- dinv[u] = (sum of the values of row u)^(-1/2): the weighted counterpart of 1 + deg_u -------------------
// Split by ENTRIES like the aggregation, so that hub rows of a power-law graph cost what their entries cost:
// a wavefront owns kSumRange consecutive entries, copies their values to LDS with coalesced loads, and then
// every lane adds up whole rows out of LDS (rows that hold more than kCoop of the range's entries are summed
// by the 64 lanes together).  A row cut by the range's ends leaves a piece in the workspace; a second small
// kernel adds a cut row's pieces in entry order.  Every sum has an order fixed by the row structure alone:
// results repeat bit for bit.
constexpr int kSumRange = 2048;
constexpr int kCoop = 64;

// p_cont: piece of the row that began in an earlier range; p_own/owner: first piece of the row that begins in
// this range and runs past its end (owner = -1: there is none)
struct SumRec { float p_cont, p_own; int32_t owner, pad; };

// Sums of eight rows at once: v[q] is this lane's share of row q.  Three exchange steps halve what a lane keeps
// (the lane's bit 0 chooses the half of q, bit 1 the quarter, bit 2 the row), three more add up over the other
// lane bits: eleven cross-lane moves instead of forty-eight.  Returns, in lane l, the sum of row l % 8.
__device__ __forceinline__ float wave_sum8(const float (&v)[8], int lane) {
    float w4[4], w2[2];
    const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4;
#pragma unroll
    for (int q = 0; q < 4; ++q) w4[q] = (b0 ? v[q + 4] : v[q]) + __shfl_xor(b0 ? v[q] : v[q + 4], 1, kWave);
#pragma unroll
    for (int q = 0; q < 2; ++q) w2[q] = (b1 ? w4[q + 2] : w4[q]) + __shfl_xor(b1 ? w4[q] : w4[q + 2], 2, kWave);
    float r = (b2 ? w2[1] : w2[0]) + __shfl_xor(b2 ? w2[0] : w2[1], 4, kWave);
    r += __shfl_xor(r, 8, kWave);
    r += __shfl_xor(r, 16, kWave);
    r += __shfl_xor(r, 32, kWave);
    // this lane now holds row 4 * bit0 + 2 * bit1 + bit2; row q is wanted in the lanes with l % 8 == q
    const int q = lane & 7;
    return __shfl(r, ((q >> 2) & 1) | (q & 2) | ((q & 1) << 2), kWave);
}

// A vertex whose row sum is not positive (no entries at all, or weights that cancel) has no normalisation; it gets
// the factor 0, so it neither sends nor receives anything, instead of an infinity that would turn into NaN.
__device__ __forceinline__ float inv_sqrt_or_zero(float s) { return s > 0.0f ? 1.0f / sqrtf(s) : 0.0f; }

__global__ __launch_bounds__(kWave) void weighted_rowsum_kernel(int n, int nnz, const int32_t *__restrict__ rowptr,
                                                               const float *__restrict__ val, SumRec *__restrict__ recs,
                                                               float *__restrict__ dinv) {
    __shared__ float s_val[kSumRange];
    const int lane = threadIdx.x, range = blockIdx.x;
    nnz = min(nnz, rowptr[n]);                          // the host's count may be an upper bound: the last row pointer decides
    const int e0 = (int)min((int64_t)range * kSumRange, (int64_t)nnz), e1 = (int)min((int64_t)e0 + kSumRange, (int64_t)nnz);
    if (e0 >= nnz && range > 0) {                       // nothing stored here
        if (lane == 0) recs[range] = SumRec{0.0f, 0.0f, -1, 0};
        return;
    }
    const bool last = e1 == nnz;
    // the values of the range, 64 consecutive ones per load
#pragma unroll 16
    for (int i = lane; i < kSumRange; i += kWave) s_val[i] = val[max(min(e0 + i, nnz - 1), 0)];   // unconditional: loads stay in flight together
    // rows of the range: the one cut by its begin (if any), then every row that begins in [e0, e1), empty ones
    // included; the last range also takes the empty rows behind the last entry
    const int k_lo = wave_find_row(rowptr, n, e0 - 1, lane) + 1;          // first row that begins at e0 or later
    const int k_first = rowptr[k_lo] > e0 ? k_lo - 1 : k_lo;              // rowptr[n] = nnz > e0
    wave_lds_sync();
    float p_cont = 0.0f, p_own = 0.0f;
    int owner = -1;
    bool more = true;
    for (int base = k_first; more; base += kWave) {
        const int r = base + lane;
        const int rb_raw = rowptr[min(r, n)];
        const bool valid = r < n && (last || rb_raw < e1);     // the range's rows end where a row begins at e1 or later
        more = __ballot(valid) == ~0ull;
        const int rb = valid ? rb_raw : e1, re = valid ? rowptr[r + 1] : e1;
        const int b = max(rb, e0) - e0, e = min(re, e1) - e0;
        const bool coop = e - b > kCoop;
        float sum = 0.0f;
        if (!coop) {                                                       // four entries a round, reads past the row's end masked
            float s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
            for (int i = b; i < e; i += 4) {
                const float x0 = s_val[i], x1 = s_val[min(i + 1, kSumRange - 1)], x2 = s_val[min(i + 2, kSumRange - 1)],
                            x3 = s_val[min(i + 3, kSumRange - 1)];
                sum += x0;
                s1 += i + 1 < e ? x1 : 0.0f;
                s2 += i + 2 < e ? x2 : 0.0f;
                s3 += i + 3 < e ? x3 : 0.0f;
            }
            sum = (sum + s1) + (s2 + s3);
        }
        // longer rows: all lanes together, eight rows per round so that one set of cross-lane moves serves eight sums
        const uint64_t coop_mask = __ballot(coop);
        const int rank = __popcll(coop_mask & ((1ull << lane) - 1));
        int group = 0;
        for (uint64_t todo = coop_mask; todo; ++group) {
            float v[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                float a0 = 0.0f, a1 = 0.0f;
                if (todo) {
                    const int src = __builtin_ctzll(todo);
                    todo &= todo - 1;
                    const int bb = __builtin_amdgcn_readlane(b, src), ee = __builtin_amdgcn_readlane(e, src);
                    int i = bb + lane;
                    for (; i + kWave < ee; i += 2 * kWave) { a0 += s_val[i]; a1 += s_val[i + kWave]; }
                    if (i < ee) a0 += s_val[i];
                }
                v[q] = a0 + a1;
            }
            const float t = __shfl(wave_sum8(v, lane), rank & 7, kWave);
            if (coop && (rank >> 3) == group) sum = t;
        }
        const bool open_l = rb < e0, open_r = re > e1;
        if (valid && !open_l && !open_r) dinv[r] = inv_sqrt_or_zero(sum);
        const uint64_t m_cont = __ballot(valid && open_l), m_own = __ballot(valid && !open_l && open_r);
        if (m_cont) p_cont = __shfl(sum, __builtin_ctzll(m_cont), kWave);
        if (m_own) { const int src = __builtin_ctzll(m_own); p_own = __shfl(sum, src, kWave); owner = base + src; }
    }
    if (lane == 0) recs[range] = SumRec{p_cont, p_own, owner, 0};
}

// a row that begins in range w and ends in a later one: its pieces in entry order
__global__ __launch_bounds__(256) void weighted_rowsum_fix_kernel(int n_ranges, const int32_t *__restrict__ rowptr,
                                                                  const SumRec *__restrict__ recs, float *__restrict__ dinv) {
    const int w = blockIdx.x * 256 + threadIdx.x;
    if (w >= n_ranges) return;
    const SumRec rec = recs[w];
    if (rec.owner < 0) return;
    const int end = rowptr[rec.owner + 1];
    float acc = rec.p_own;
    for (int r = w + 1; (int64_t)r * kSumRange < end; ++r) acc += recs[r].p_cont;
    dinv[rec.owner] = inv_sqrt_or_zero(acc);
}

size_t weighted_dinv_workspace(int64_t nnz) {
    return round_up(sizeof(SumRec) * (size_t)((nnz + kSumRange - 1) / kSumRange), (size_t)256) + 256;
}

}  // namespace

extern "C" int dgnn_csr_weighted_dinv_workspace(int64_t nnz, size_t *bytes) {
    if (!bytes) return DGNN_ERR_NULL;
    if (nnz < 0) return DGNN_ERR_SHAPE;
    if (!fits_index(nnz)) return DGNN_ERR_OVERFLOW;
    *bytes = weighted_dinv_workspace(nnz);
    return DGNN_OK;
}

extern "C" int dgnn_csr_weighted_dinv(int64_t n, int64_t nnz, const int32_t *rowptr, const float *val, float *dinv,
                                      void *ws, size_t ws_bytes, void *stream) {
    if (!rowptr || !val || !dinv || !ws) return DGNN_ERR_NULL;
    if (n <= 0 || nnz <= 0) return DGNN_ERR_SHAPE;
    if (!fits_index(n + 1) || !fits_index(nnz)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(ws)) return DGNN_ERR_ALIGN;
    if (ws_bytes < weighted_dinv_workspace(nnz)) return DGNN_ERR_CAPACITY;
    hipStream_t s = (hipStream_t)stream;
    const int ranges = (int)((nnz + kSumRange - 1) / kSumRange);
    hipLaunchKernelGGL(weighted_rowsum_kernel, dim3((unsigned)ranges), dim3(kWave), 0, s, (int)n, (int)nnz, rowptr, val,
                       (SumRec *)ws, dinv);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    hipLaunchKernelGGL(weighted_rowsum_fix_kernel, dim3((unsigned)((ranges + 255) / 256)), dim3(256), 0, s, ranges, rowptr,
                       (const SumRec *)ws, dinv);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}
