// Sparse factor of the GCN operation, Eqn (1) and Eqn (2): Z = sigma?(A~ H) with
// A~ = D^(-1/2) (A + I) D^(-1/2).  The snapshot is unweighted, so a stored entry (u, v) weighs
// dinv[u] * dinv[v] and the kernel needs no value array:
//     Z[u] = dinv[u] * sum_{v in row u} dinv[v] * H[v].
//
// The work is a gather of whole H rows (one 16-byte piece per lane, a lane group per row of H),
// bound by how many independent row fetches are in flight, so it is split by ENTRIES, not by
// rows: a workgroup owns a tile of consecutive stored entries, whatever rows they belong to.
//   1. Two wavefronts find the rows that hold the first and the last entry of the tile (64-ary
//      search), the others stage the tile's column indices (and dinv of the columns) in LDS.
//   2. Row starts inside the tile are scattered into LDS and max-scanned into a row id per entry.
//   3. Every lane group walks the same number of consecutive entries, eight gathers in flight at
//      a time, and flushes its running sum whenever the row id changes: a row segment that
//      begins and ends inside the group's range is a finished row and is stored at once; a
//      segment cut by the range is parked in LDS.
//   4. One lane group adds the parked pieces up in entry order.  Rows cut by the tile itself
//      leave a "left" and/or "right" carry in the workspace; a second small kernel adds the
//      carries of consecutive tiles, again in entry order.
// Hub rows of power-law graphs are thereby spread over as many workgroups as they have tiles,
// short rows share a wavefront, and every sum has a fixed order: no floating-point atomics,
// results repeat bit for bit.
#include "common.hpp"

namespace {

using namespace dgnn;

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kBatch = 8;          // gathers issued together by a lane group
constexpr int kMaxTile = 2048;     // entries per tile, upper limit (LDS)

enum : int32_t { kLeft = 1, kLeftClosed = 2, kRight = 4 };
struct TileRec { int32_t flags, row_first, row_last, pad; };

template <int LPR> struct Shape {
    static constexpr int kGroups = kThreads / LPR;
    static constexpr int kTile = kGroups * 32 > kMaxTile ? kMaxTile : kGroups * 32;
    static constexpr int kPerGroup = kTile / kGroups;      // entries walked by one lane group
    static constexpr int kItems = kTile / kThreads;        // entries per thread in the scan
};

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
        *static_cast<floatx4 *>(p) = floatx4{acc[0], acc[1], acc[2], acc[3]};
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
        *static_cast<uintx4 *>(p) = v;
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

// SCALE_V: multiply every gathered row by dinv of its column (otherwise H already carries it).
template <int LPR, bool BF16, bool SCALE_V>
__global__ __launch_bounds__(kThreads) void spmm_tile_kernel(
    int n, int nnz, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const float *__restrict__ dinv, const char *__restrict__ h, char *__restrict__ z, int relu,
    TileRec *__restrict__ recs, float *__restrict__ carry) {
    typedef Shape<LPR> S;
    typedef typename Piece<BF16>::Raw Raw;
    constexpr int NV = Piece<BF16>::kVals;
    constexpr int F = LPR * NV;
    constexpr int G = S::kGroups, TILE = S::kTile, PER = S::kPerGroup, ITEMS = S::kItems;
    constexpr int kRowBytes = LPR * 16;

    __shared__ int s_col[TILE];
    __shared__ int s_rid[TILE];
    __shared__ float s_dv[SCALE_V ? TILE : 1];
    __shared__ float s_part[G][2][F];
    __shared__ int s_flag[G];
    __shared__ int s_prow[G][2];
    __shared__ int s_rows[2];
    __shared__ int s_wmax[kThreads / kWave];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int i0 = (int)((int64_t)blockIdx.x * TILE);
    const int i1 = (int)min((int64_t)i0 + TILE, (int64_t)nnz);
    const int cnt = i1 - i0;

    // ---- 1. stage the tile; meanwhile two wavefronts look up the bounding rows
    int myc[ITEMS];
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        const int p = tid + k * kThreads;
        myc[k] = p < cnt ? colidx[i0 + p] : 0;
    }
    if (wave < 2) {
        int r = wave_find_row(rowptr, n, wave == 0 ? i0 : i1 - 1, lane);
        if (lane == 0) s_rows[wave] = max(r, 0);
    }
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        const int p = tid + k * kThreads;
        s_rid[p] = 0;
        s_col[p] = myc[k];
        if (SCALE_V) s_dv[p] = p < cnt ? dinv[myc[k]] : 0.0f;
    }
    __syncthreads();
    const int r_first = s_rows[0], r_last = s_rows[1];
    const bool first_open = rowptr[r_first] < i0;        // the tile's first row began in an earlier tile
    const bool last_open = rowptr[r_last + 1] > i1;      // its last row goes on in a later tile

    // ---- 2. row id (relative to r_first) of every entry
    for (int k = r_first + 1 + tid; k <= r_last; k += kThreads) {
        const int a = rowptr[k], b = rowptr[k + 1];
        const unsigned p = (unsigned)(a - i0);
        if (a == b) {                                    // a row without entries: its output is zero
            float zero[NV];
#pragma unroll
            for (int q = 0; q < NV; ++q) zero[q] = 0.0f;
            for (int sub = 0; sub < LPR; ++sub) Piece<BF16>::store(z + (int64_t)k * kRowBytes + sub * 16, zero);
        } else if (p < (unsigned)cnt) {
            atomicMax(&s_rid[p], k - r_first);
        }
    }
    __syncthreads();
    {
        int v[ITEMS];
        int m = 0;
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
            m = max(m, s_rid[tid * ITEMS + k]);
            v[k] = m;
        }
        const int inc = wave_scan_max(m, lane);
        if (lane == kWave - 1) s_wmax[wave] = inc;
        int before = __shfl_up(inc, 1, kWave);
        if (lane == 0) before = 0;
        __syncthreads();
        for (int w = 0; w < wave; ++w) before = max(before, s_wmax[w]);
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) s_rid[tid * ITEMS + k] = max(v[k], before);
    }
    __syncthreads();

    // ---- 3. every lane group walks PER consecutive entries
    const int g = tid / LPR, sub = tid % LPR;
    const int c0 = g * PER;
    const int c1 = min(c0 + PER, cnt);
    int flags = 0;
    if (c0 < c1) {
        int cur = s_rid[c0];
        // is the first segment of this range the beginning of its row?
        bool left_closed = c0 == 0 ? !first_open : s_rid[c0 - 1] != cur;
        float acc[NV];
#pragma unroll
        for (int q = 0; q < NV; ++q) acc[q] = 0.0f;

        auto flush = [&](bool right_closed) {
            if (left_closed && right_closed) {
                finish_row<BF16, NV>(z, (int64_t)r_first + cur, kRowBytes, sub, dinv, relu, acc);
            } else {
                const int slot = left_closed ? 1 : 0;    // 0: cut on the left, 1: cut on the right only
#pragma unroll
                for (int q = 0; q < NV; ++q) s_part[g][slot][sub * NV + q] = acc[q];
                if (sub == 0) s_prow[g][slot] = cur;
                flags |= left_closed ? kRight : (kLeft | (right_closed ? kLeftClosed : 0));
            }
        };

#pragma unroll
        for (int b = 0; b < PER / kBatch; ++b) {
            const int p0 = c0 + b * kBatch;
            Raw raw[kBatch];
            int rid[kBatch];
            float dv[kBatch];
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                const int p = p0 + k;
                if (p < c1) {
                    rid[k] = s_rid[p];
                    dv[k] = SCALE_V ? s_dv[p] : 1.0f;
                    raw[k] = *reinterpret_cast<const Raw *>(h + (int64_t)s_col[p] * kRowBytes + sub * 16);
                }
            }
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                if (p0 + k < c1) {
                    if (rid[k] != cur) {
                        flush(true);
                        left_closed = true;
                        cur = rid[k];
#pragma unroll
                        for (int q = 0; q < NV; ++q) acc[q] = 0.0f;
                    }
                    Piece<BF16>::fma(acc, dv[k], raw[k]);
                }
            }
        }
        flush(c1 == cnt ? !last_open : s_rid[c1] != cur);
    }
    if (sub == 0) s_flag[g] = flags;
    __syncthreads();

    // ---- 4. one lane group adds the parked pieces in entry order
    if (tid < LPR) {
        float acc[NV];
#pragma unroll
        for (int q = 0; q < NV; ++q) acc[q] = 0.0f;
        bool running = false;      // a row is being accumulated
        bool began_here = false;   // ... and it began inside this tile
        int run_row = 0;
        int tile_flags = 0;
        float *my_carry = carry + (int64_t)blockIdx.x * 2 * F;
        for (int gg = 0; gg < G; ++gg) {
            const int fl = s_flag[gg];
            if (fl & kLeft) {
#pragma unroll
                for (int q = 0; q < NV; ++q) acc[q] += s_part[gg][0][tid * NV + q];
                if (!running) { running = true; began_here = false; run_row = s_prow[gg][0]; }
                if (fl & kLeftClosed) {
                    if (began_here) {
                        finish_row<BF16, NV>(z, (int64_t)r_first + run_row, kRowBytes, tid, dinv, relu, acc);
                    } else {                         // end of the row inherited from the previous tile
#pragma unroll
                        for (int q = 0; q < NV; ++q) my_carry[tid * NV + q] = acc[q];
                        tile_flags |= kLeft | kLeftClosed;
                    }
                    running = false;
#pragma unroll
                    for (int q = 0; q < NV; ++q) acc[q] = 0.0f;
                }
            }
            if (fl & kRight) {
#pragma unroll
                for (int q = 0; q < NV; ++q) acc[q] = s_part[gg][1][tid * NV + q];
                running = true;
                began_here = true;
                run_row = s_prow[gg][1];
            }
        }
        if (running) {
            if (began_here) {                        // goes on in the next tile
#pragma unroll
                for (int q = 0; q < NV; ++q) my_carry[F + tid * NV + q] = acc[q];
                tile_flags |= kRight;
            } else {                                 // the whole tile lies inside one row
#pragma unroll
                for (int q = 0; q < NV; ++q) my_carry[tid * NV + q] = acc[q];
                tile_flags |= kLeft;
            }
        }
        if (tid == 0) recs[blockIdx.x] = TileRec{tile_flags, r_first, r_last, 0};
    }

    // rows without entries just before this tile's first row and after the last stored entry (there are
    // none when every row holds its diagonal); rows without entries inside the tile were zeroed above
    {
        float zero[NV];
#pragma unroll
        for (int q = 0; q < NV; ++q) zero[q] = 0.0f;
        if (!first_open)
            for (int k = r_first - 1 - tid; k >= 0; k -= kThreads) {
                if (rowptr[k] != i0) break;
                for (int q = 0; q < LPR; ++q) Piece<BF16>::store(z + (int64_t)k * kRowBytes + q * 16, zero);
            }
        if (i1 == nnz)
            for (int k = r_last + 1 + tid; k < n; k += kThreads)
                for (int q = 0; q < LPR; ++q) Piece<BF16>::store(z + (int64_t)k * kRowBytes + q * 16, zero);
    }
}

// Rows cut by tile boundaries: the tile where such a row begins owns it and adds the left carries
// of the following tiles until the one that closes the row.
template <int LPR, bool BF16>
__global__ __launch_bounds__(kThreads) void spmm_carry_kernel(int tiles, const TileRec *__restrict__ recs,
                                                              const float *__restrict__ carry,
                                                              const float *__restrict__ dinv, char *__restrict__ z, int relu) {
    constexpr int NV = Piece<BF16>::kVals;
    constexpr int F = LPR * NV;
    constexpr int G = kThreads / LPR;
    const int tid = threadIdx.x;
    const int sub = tid % LPR;
    const int t = blockIdx.x * G + tid / LPR;
    if (t >= tiles) return;
    const TileRec rec = recs[t];
    if (!(rec.flags & kRight)) return;
    float acc[NV];
#pragma unroll
    for (int q = 0; q < NV; ++q) acc[q] = carry[((int64_t)t * 2 + 1) * F + sub * NV + q];
    for (int j = t + 1; j < tiles; ++j) {
        const int fj = recs[j].flags;
        if (!(fj & kLeft)) break;
#pragma unroll
        for (int q = 0; q < NV; ++q) acc[q] += carry[(int64_t)j * 2 * F + sub * NV + q];
        if (fj & kLeftClosed) break;
    }
    finish_row<BF16, NV>(z, (int64_t)rec.row_last, LPR * 16, sub, dinv, relu, acc);
}

struct Workspace {
    TileRec *recs;
    float *carry;
};

// Sized for the smallest tile a width can get (fp32 storage), so one query serves both dtypes.
size_t workspace_layout(int64_t nnz, int32_t f, Workspace *ws, void *base) {
    const int lpr = f / 4;
    const int groups = kThreads / lpr;
    const int tile = groups * 32 > kMaxTile ? kMaxTile : groups * 32;
    const int64_t tiles = (nnz + tile - 1) / tile + 1;
    const size_t o_recs = 0;
    const size_t o_carry = round_up((size_t)tiles * sizeof(TileRec), 256);
    const size_t total = o_carry + round_up((size_t)tiles * 2 * f * sizeof(float), 256);
    if (ws) {
        char *b = static_cast<char *>(base);
        ws->recs = reinterpret_cast<TileRec *>(b + o_recs);
        ws->carry = reinterpret_cast<float *>(b + o_carry);
    }
    return total;
}

template <int LPR, bool BF16>
int launch(int64_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *dinv, bool scale_v,
           const void *h, void *z, int relu, const Workspace &ws, hipStream_t s) {
    constexpr int TILE = Shape<LPR>::kTile;
    constexpr int G = kThreads / LPR;
    const int tiles = (int)((nnz + TILE - 1) / TILE);
    if (tiles == 0) return DGNN_ERR_SHAPE;
    if (scale_v)
        hipLaunchKernelGGL((spmm_tile_kernel<LPR, BF16, true>), dim3(tiles), dim3(kThreads), 0, s, (int)n, (int)nnz, rowptr,
                           colidx, dinv, static_cast<const char *>(h), static_cast<char *>(z), relu, ws.recs, ws.carry);
    else
        hipLaunchKernelGGL((spmm_tile_kernel<LPR, BF16, false>), dim3(tiles), dim3(kThreads), 0, s, (int)n, (int)nnz, rowptr,
                           colidx, dinv, static_cast<const char *>(h), static_cast<char *>(z), relu, ws.recs, ws.carry);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    hipLaunchKernelGGL((spmm_carry_kernel<LPR, BF16>), dim3((tiles + G - 1) / G), dim3(kThreads), 0, s, tiles, ws.recs,
                       ws.carry, dinv, static_cast<char *>(z), relu);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

}  // namespace

extern "C" int dgnn_spmm_workspace(int64_t n, int64_t nnz, int32_t f, size_t *bytes) {
    if (!bytes) return DGNN_ERR_NULL;
    if (n <= 0 || nnz < 0 || !supported_width(f)) return DGNN_ERR_SHAPE;
    if (!fits_i32(n + 1) || !fits_i32(nnz)) return DGNN_ERR_OVERFLOW;
    *bytes = workspace_layout(nnz, f, nullptr, nullptr);
    return DGNN_OK;
}

extern "C" int dgnn_spmm(int64_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *dinv,
                         const void *h, int32_t f, void *z, dgnn_dtype dt, uint32_t flags,
                         void *ws, size_t ws_bytes, void *stream) {
    if (!rowptr || !colidx || !h || !z || !ws) return DGNN_ERR_NULL;
    if (n <= 0 || nnz <= 0 || !supported_width(f) || (flags & ~(DGNN_RELU | DGNN_H_PRESCALED))) return DGNN_ERR_SHAPE;
    if (dt != DGNN_F32 && dt != DGNN_BF16) return DGNN_ERR_SHAPE;
    if (!fits_i32(n + 1) || !fits_i32(nnz)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(h) || !aligned16(z) || !aligned16(ws)) return DGNN_ERR_ALIGN;
    if (h == z) return DGNN_ERR_ALIAS;
    Workspace w;
    if (ws_bytes < workspace_layout(nnz, f, &w, ws)) return DGNN_ERR_CAPACITY;
    hipStream_t s = (hipStream_t)stream;
    const int relu = (flags & DGNN_RELU) ? 1 : 0;
    const bool scale_v = dinv != nullptr && !(flags & DGNN_H_PRESCALED);
    const int lpr = dt == DGNN_F32 ? f / 4 : f / 8;   // lanes per feature row, 16 bytes each
    const bool bf = dt == DGNN_BF16;
    switch (lpr) {
        case 2: return launch<2, true>(n, nnz, rowptr, colidx, dinv, scale_v, h, z, relu, w, s);
        case 4: return bf ? launch<4, true>(n, nnz, rowptr, colidx, dinv, scale_v, h, z, relu, w, s)
                          : launch<4, false>(n, nnz, rowptr, colidx, dinv, scale_v, h, z, relu, w, s);
        case 8: return bf ? launch<8, true>(n, nnz, rowptr, colidx, dinv, scale_v, h, z, relu, w, s)
                          : launch<8, false>(n, nnz, rowptr, colidx, dinv, scale_v, h, z, relu, w, s);
        case 16: return bf ? launch<16, true>(n, nnz, rowptr, colidx, dinv, scale_v, h, z, relu, w, s)
                           : launch<16, false>(n, nnz, rowptr, colidx, dinv, scale_v, h, z, relu, w, s);
        case 32: return launch<32, false>(n, nnz, rowptr, colidx, dinv, scale_v, h, z, relu, w, s);
        default: return DGNN_ERR_SHAPE;
    }
}
