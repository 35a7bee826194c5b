// Sparse factor of the GCN operation, Eqn (1) and Eqn (2): Z = sigma?(A~ H) with
// A~ = D^(-1/2) (A + I) D^(-1/2).  The snapshot is unweighted, so a stored entry (u, v) weighs
// dinv[u] * dinv[v] and the kernel needs no value array:
//     Z[u] = dinv[u] * sum_{v in row u} dinv[v] * H[v].
//
// The work is a gather of whole H rows (one 16-byte piece per lane), bound by how many
// independent row fetches are in flight.  Rows are binned by length:
//   short rows (<= kLongRow entries)  one lane group per row (group = F*s/16 lanes), several
//                                     rows per wavefront, a full group-width of gathers in
//                                     flight per step;
//   long rows  (>  kLongRow)          found by the short-row kernel, which appends them to a
//                                     list in the workspace; they are cut into chunks of kChunk
//                                     entries, one wavefront per chunk, and the per-chunk
//                                     partial sums are added up in chunk order by a last kernel.
// No floating-point atomics: the order of every sum is fixed, so results repeat bit for bit.
#include "common.hpp"

namespace {

using namespace dgnn;

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kLongRow = 512;     // rows longer than this leave the lane-group path
constexpr int kChunk = 1024;      // entries of a long row handled by one wavefront
constexpr int kLongGrid = 2048;   // workgroups of the long-row kernels (they loop)

struct Header {          // first 16 bytes of the workspace
    int32_t n_items;     // chunks of long rows
    int32_t n_long;      // long rows
    int32_t pad[2];
};
struct LongRow { int32_t row, first_item, n_items, pad; };
struct Item { int32_t long_slot, chunk; };

struct Workspace {
    Header *hdr;
    LongRow *rows;
    Item *items;
    float *partial;
    int32_t max_long, max_items;
};

size_t workspace_layout(int64_t nnz, int32_t f, Workspace *ws, void *base) {
    int64_t max_long = nnz / kLongRow + 1;
    int64_t max_items = nnz / kChunk + max_long + 1;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += round_up(bytes, 256); return o; };
    size_t o_hdr = take(sizeof(Header));
    size_t o_rows = take((size_t)max_long * sizeof(LongRow));
    size_t o_items = take((size_t)max_items * sizeof(Item));
    size_t o_part = take((size_t)max_items * f * sizeof(float));
    if (ws) {
        char *b = static_cast<char *>(base);
        ws->hdr = reinterpret_cast<Header *>(b + o_hdr);
        ws->rows = reinterpret_cast<LongRow *>(b + o_rows);
        ws->items = reinterpret_cast<Item *>(b + o_items);
        ws->partial = reinterpret_cast<float *>(b + o_part);
        ws->max_long = (int32_t)max_long;
        ws->max_items = (int32_t)max_items;
    }
    return off;
}

// ---- 16-byte feature pieces: 4 fp32 or 8 bf16, accumulated in fp32 -------------------------
template <bool BF16> struct Piece;
template <> struct Piece<false> {
    static constexpr int kVals = 4;
    static __device__ __forceinline__ void fma(float (&acc)[4], float s, const void *p) {
        floatx4 v = *static_cast<const floatx4 *>(p);
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] = fmaf(s, v[e], acc[e]);
    }
    static __device__ __forceinline__ void store(void *p, const float (&acc)[4]) {
        *static_cast<floatx4 *>(p) = floatx4{acc[0], acc[1], acc[2], acc[3]};
    }
};
template <> struct Piece<true> {
    static constexpr int kVals = 8;
    static __device__ __forceinline__ void fma(float (&acc)[8], float s, const void *p) {
        uintx4 v = *static_cast<const uintx4 *>(p);
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

__global__ void reset_kernel(Header *hdr) {
    if (threadIdx.x == 0 && blockIdx.x == 0) { hdr->n_items = 0; hdr->n_long = 0; }
}

// One lane group (LPR lanes, 16 bytes of the feature row each) per short row.
template <int LPR, bool BF16>
__global__ __launch_bounds__(kThreads) void spmm_short_kernel(
    int n, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx, const float *__restrict__ dinv,
    const char *__restrict__ h, char *__restrict__ z, int relu, Workspace ws) {
    constexpr int NV = Piece<BF16>::kVals;
    constexpr int kRowBytes = LPR * 16;
    constexpr int kGroups = kThreads / LPR;
    const int tid = threadIdx.x;
    const int sub = tid % LPR;
    const int lane = tid & (kWave - 1);
    const int gbase = lane - sub;                  // first lane of this group inside the wavefront
    const int64_t u = (int64_t)blockIdx.x * kGroups + tid / LPR;
    if (u >= n) return;
    const int s = rowptr[u], e = rowptr[u + 1];
    if (e - s > kLongRow) {
        if (sub == 0) {
            int nch = (e - s + kChunk - 1) / kChunk;
            int slot = atomicAdd(&ws.hdr->n_long, 1);
            int first = atomicAdd(&ws.hdr->n_items, nch);
            if (slot < ws.max_long && first + nch <= ws.max_items) {
                ws.rows[slot] = LongRow{(int32_t)u, first, nch, 0};
                for (int k = 0; k < nch; ++k) ws.items[first + k] = Item{slot, k};
            }
        }
        return;
    }
    float acc[NV];
#pragma unroll
    for (int q = 0; q < NV; ++q) acc[q] = 0.0f;
    for (int p = s; p < e; p += LPR) {
        int myc = 0;
        float myd = 0.0f;
        if (p + sub < e) {
            myc = colidx[p + sub];
            myd = dinv ? dinv[myc] : 1.0f;
        }
#pragma unroll
        for (int k = 0; k < LPR; ++k) {
            int c = __shfl(myc, gbase + k, kWave);
            float d = __shfl(myd, gbase + k, kWave);
            if (p + k < e) Piece<BF16>::fma(acc, d, h + (int64_t)c * kRowBytes + sub * 16);
        }
    }
    const float du = dinv ? dinv[u] : 1.0f;
#pragma unroll
    for (int q = 0; q < NV; ++q) {
        acc[q] *= du;
        if (relu) acc[q] = fmaxf(acc[q], 0.0f);
    }
    Piece<BF16>::store(z + u * kRowBytes + sub * 16, acc);
}

// One wavefront per chunk of a long row; the 64 / LPR groups of the wavefront take entries in
// turn and are then folded together with a fixed butterfly.
template <int LPR, bool BF16>
__global__ __launch_bounds__(kThreads) void spmm_long_kernel(
    const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx, const float *__restrict__ dinv,
    const char *__restrict__ h, Workspace ws) {
    constexpr int NV = Piece<BF16>::kVals;
    constexpr int kRowBytes = LPR * 16;
    constexpr int kGroupsPerWave = kWave / LPR;
    constexpr int F = LPR * NV;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int sub = lane % LPR, grp = lane / LPR;
    const int n_items = min(ws.hdr->n_items, ws.max_items);
    const int wave_global = blockIdx.x * (kThreads / kWave) + tid / kWave;
    const int wave_count = gridDim.x * (kThreads / kWave);
    for (int it = wave_global; it < n_items; it += wave_count) {
        const Item item = ws.items[it];
        const LongRow lr = ws.rows[item.long_slot];
        const int s = rowptr[lr.row] + item.chunk * kChunk;
        const int e = min(s + kChunk, rowptr[lr.row + 1]);
        float acc[NV];
#pragma unroll
        for (int q = 0; q < NV; ++q) acc[q] = 0.0f;
        // each pass of the wavefront covers 64 entries: lane l fetches index and dinv of entry
        // p + l, then group g accumulates entries p + g, p + g + G, ...
        for (int p = s; p < e; p += kWave) {
            int myc = 0;
            float myd = 0.0f;
            if (p + lane < e) {
                myc = colidx[p + lane];
                myd = dinv ? dinv[myc] : 1.0f;
            }
#pragma unroll
            for (int k = 0; k < LPR; ++k) {
                const int src = k * kGroupsPerWave + grp;
                int c = __shfl(myc, src, kWave);
                float d = __shfl(myd, src, kWave);
                if (p + src < e) Piece<BF16>::fma(acc, d, h + (int64_t)c * kRowBytes + sub * 16);
            }
        }
#pragma unroll
        for (int off = LPR; off < kWave; off <<= 1) {
#pragma unroll
            for (int q = 0; q < NV; ++q) acc[q] += __shfl_xor(acc[q], off, kWave);
        }
        if (grp == 0) {
            float *dst = ws.partial + (int64_t)it * F + sub * NV;
#pragma unroll
            for (int q = 0; q < NV; ++q) dst[q] = acc[q];
        }
    }
}

// One lane group per long row: partial sums added in chunk order, then scale, sigma, store.
template <int LPR, bool BF16>
__global__ __launch_bounds__(kThreads) void spmm_long_reduce_kernel(const float *__restrict__ dinv,
                                                                    char *__restrict__ z, int relu, Workspace ws) {
    constexpr int NV = Piece<BF16>::kVals;
    constexpr int kRowBytes = LPR * 16;
    constexpr int kGroups = kThreads / LPR;
    constexpr int F = LPR * NV;
    const int tid = threadIdx.x;
    const int sub = tid % LPR;
    const int n_long = min(ws.hdr->n_long, ws.max_long);
    for (int slot = blockIdx.x * kGroups + tid / LPR; slot < n_long; slot += gridDim.x * kGroups) {
        const LongRow lr = ws.rows[slot];
        float acc[NV];
#pragma unroll
        for (int q = 0; q < NV; ++q) acc[q] = 0.0f;
        for (int k = 0; k < lr.n_items; ++k) {
            const float *src = ws.partial + (int64_t)(lr.first_item + k) * F + sub * NV;
#pragma unroll
            for (int q = 0; q < NV; ++q) acc[q] += src[q];
        }
        const float du = dinv ? dinv[lr.row] : 1.0f;
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            acc[q] *= du;
            if (relu) acc[q] = fmaxf(acc[q], 0.0f);
        }
        Piece<BF16>::store(z + (int64_t)lr.row * kRowBytes + sub * 16, acc);
    }
}

template <int LPR, bool BF16>
int launch(int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *dinv, const void *h, void *z,
           int relu, const Workspace &ws, hipStream_t s) {
    constexpr int kGroups = kThreads / LPR;
    hipLaunchKernelGGL(reset_kernel, dim3(1), dim3(64), 0, s, ws.hdr);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    hipLaunchKernelGGL((spmm_short_kernel<LPR, BF16>), dim3((unsigned)((n + kGroups - 1) / kGroups)), dim3(kThreads), 0, s,
                       (int)n, rowptr, colidx, dinv, static_cast<const char *>(h), static_cast<char *>(z), relu, ws);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    hipLaunchKernelGGL((spmm_long_kernel<LPR, BF16>), dim3(kLongGrid), dim3(kThreads), 0, s,
                       rowptr, colidx, dinv, static_cast<const char *>(h), ws);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    hipLaunchKernelGGL((spmm_long_reduce_kernel<LPR, BF16>), dim3(256), dim3(kThreads), 0, s,
                       dinv, static_cast<char *>(z), relu, ws);
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
    if (n <= 0 || nnz < 0 || !supported_width(f) || (flags & ~DGNN_RELU)) return DGNN_ERR_SHAPE;
    if (dt != DGNN_F32 && dt != DGNN_BF16) return DGNN_ERR_SHAPE;
    if (!fits_i32(n + 1) || !fits_i32(nnz)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(h) || !aligned16(z) || !aligned16(ws)) return DGNN_ERR_ALIGN;
    if (h == z) return DGNN_ERR_ALIAS;
    Workspace w;
    if (ws_bytes < workspace_layout(nnz, f, &w, ws)) return DGNN_ERR_CAPACITY;
    hipStream_t s = (hipStream_t)stream;
    const int relu = (flags & DGNN_RELU) ? 1 : 0;
    const int lpr = dt == DGNN_F32 ? f / 4 : f / 8;   // lanes per feature row, 16 bytes each
    const bool bf = dt == DGNN_BF16;
    switch (lpr) {
        case 2: return launch<2, true>(n, rowptr, colidx, dinv, h, z, relu, w, s);
        case 4: return bf ? launch<4, true>(n, rowptr, colidx, dinv, h, z, relu, w, s)
                          : launch<4, false>(n, rowptr, colidx, dinv, h, z, relu, w, s);
        case 8: return bf ? launch<8, true>(n, rowptr, colidx, dinv, h, z, relu, w, s)
                          : launch<8, false>(n, rowptr, colidx, dinv, h, z, relu, w, s);
        case 16: return bf ? launch<16, true>(n, rowptr, colidx, dinv, h, z, relu, w, s)
                           : launch<16, false>(n, rowptr, colidx, dinv, h, z, relu, w, s);
        case 32: return launch<32, false>(n, rowptr, colidx, dinv, h, z, relu, w, s);
        default: return DGNN_ERR_SHAPE;
    }
}
