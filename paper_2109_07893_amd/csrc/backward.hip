// Gradient propagation through the GCN operation of Eqn (2) (Section "Gradient Checkpoint": after a block
// has been run forward again, gradients travel through it in the reverse direction).  With
//     H = X W,   P = A~ H,   Z = max(P, 0)
// and G_Z = dL/dZ arriving from the layer above (or from the adjoint of the M-transform):
//     G_P = G_Z where Z > 0, else 0              relu_backward_kernel (can fold a row scale in)
//     G_H = A~^T G_P                              the aggregation kernel on the transposed snapshot
//     dW  = X^T G_H                               wgrad_kernel + wgrad_reduce_kernel   (this file)
//     dX  = G_H W^T                               the X W kernels with W read transposed
//
// dW = X^T G_H contracts over the N rows, so it reads both matrices once (HBM-bound, 2 s N F bytes) and
// leaves an F x F' result.  The rows are dealt out in steps of 16 to "row workers"; a worker keeps its
// part of the F x F' accumulator in MFMA registers for its whole share of the rows.  In a 32x32xK MFMA
// lane (i, h) supplies A[i][k-slice h] and B[k-slice h][i]; with A = X^T and B = G_H both operands of a
// lane are elements of column i of a 32-column tile, taken from the rows of the k-slice, which are plain
// strided loads (whole 128-byte or 64-byte runs per row across the lanes), no transposition needed.
// Workers write their partial results to the workspace and a second kernel adds them up in a fixed order,
// so the result repeats bit for bit (no floating-point atomics).
#include <algorithm>
#include <type_traits>

#include "common.hpp"

namespace {

using namespace dgnn;

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / kWave;
constexpr int kStepRows = 16;        // rows per step: eight fp32 MFMAs of depth 2, or one bf16 MFMA of depth 16
constexpr int kMaxBlocks = 512;      // two workgroups per compute unit keep enough loads in flight; bounds the workspace

// How the 32x32 tiles of the F x F' accumulator are shared out inside a workgroup: a wavefront holds
// TI x TJ tiles (at most four), GROUPS wavefronts cover all tiles, and the remaining factor of the four
// wavefronts splits the rows (RS row workers per workgroup).
template <int FIN, int FOUT>
struct Split {
    static constexpr int NI = (FIN + 31) / 32, NJ = (FOUT + 31) / 32;
    static constexpr int TILES = NI * NJ;
    static constexpr int TPW = TILES < 4 ? TILES : 4;
    static constexpr int TI = (NI >= 2 && NJ >= 2) ? 2 : (NI < TPW ? NI : TPW);
    static constexpr int TJ = TPW / TI;
    static constexpr int GI = NI / TI, GJ = NJ / TJ;
    static constexpr int GROUPS = GI * GJ;
    static constexpr int RS = kWavesPerBlock / GROUPS;
    static_assert(TI * TJ == TPW && GI * TI == NI && GJ * TJ == NJ && RS * GROUPS == kWavesPerBlock, "tile split");
};

template <int FIN, int FOUT, bool BF16>
__global__ __launch_bounds__(kThreads) void wgrad_kernel(const void *__restrict__ xv, const void *__restrict__ gv, int64_t n,
                                                         int64_t n_steps, float *__restrict__ partial) {
    using S = Split<FIN, FOUT>;
    typedef typename std::conditional<BF16, uint16_t, float>::type Elem;
    typedef typename std::conditional<BF16, uint32_t, float>::type Raw;
    const Elem *x = static_cast<const Elem *>(xv);
    const Elem *g = static_cast<const Elem *>(gv);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int i = lane & 31, hh = lane >> 5;
    const int group = wave % S::GROUPS, rs = wave / S::GROUPS;
    const int it0 = (group / S::GJ) * S::TI, jt0 = (group % S::GJ) * S::TJ;
    const int64_t workers = (int64_t)gridDim.x * S::RS;
    const int64_t me = (int64_t)blockIdx.x * S::RS + rs;

    floatx16 acc[S::TI][S::TJ];
#pragma unroll
    for (int ti = 0; ti < S::TI; ++ti)
#pragma unroll
        for (int tj = 0; tj < S::TJ; ++tj)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ti][tj][v] = 0.0f;

    // Row of the k-slice element e of this lane inside a step: depth-2 MFMAs take rows (2 e + h), the
    // depth-16 MFMA takes rows (8 h + e).
    auto row_of = [&](int64_t step, int e) { return step * kStepRows + (BF16 ? 8 * hh + e : 2 * e + hh); };
    // Loads are unconditional (addresses clamped into the matrices); what lies outside is zeroed when used.
    Raw xa_next[S::TI][8], gb_next[S::TJ][8];
    auto fetch = [&](int64_t step) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int64_t row = std::min<int64_t>(row_of(step, e), n - 1);
#pragma unroll
            for (int ti = 0; ti < S::TI; ++ti) xa_next[ti][e] = x[row * FIN + std::min((it0 + ti) * 32 + i, FIN - 1)];
#pragma unroll
            for (int tj = 0; tj < S::TJ; ++tj) gb_next[tj][e] = g[row * FOUT + std::min((jt0 + tj) * 32 + i, FOUT - 1)];
        }
    };
    if (me < n_steps) fetch(me);
    for (int64_t step = me; step < n_steps; step += workers) {
        Raw xa[S::TI][8], gb[S::TJ][8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const bool row_ok = row_of(step, e) < n;
#pragma unroll
            for (int ti = 0; ti < S::TI; ++ti) xa[ti][e] = (row_ok && (it0 + ti) * 32 + i < FIN) ? xa_next[ti][e] : Raw(0);
#pragma unroll
            for (int tj = 0; tj < S::TJ; ++tj) gb[tj][e] = (row_ok && (jt0 + tj) * 32 + i < FOUT) ? gb_next[tj][e] : Raw(0);
        }
        fetch(std::min(step + workers, n_steps - 1));      // the next step's rows travel while this one is multiplied
        __builtin_amdgcn_sched_barrier(0);                  // ... so the loads must stay ahead of the multiplications
        if constexpr (BF16) {
            bf16x8 a[S::TI], b[S::TJ];
#pragma unroll
            for (int ti = 0; ti < S::TI; ++ti) {
                const uintx4 p = {xa[ti][0] | (xa[ti][1] << 16), xa[ti][2] | (xa[ti][3] << 16), xa[ti][4] | (xa[ti][5] << 16),
                                  xa[ti][6] | (xa[ti][7] << 16)};
                a[ti] = __builtin_bit_cast(bf16x8, p);
            }
#pragma unroll
            for (int tj = 0; tj < S::TJ; ++tj) {
                const uintx4 p = {gb[tj][0] | (gb[tj][1] << 16), gb[tj][2] | (gb[tj][3] << 16), gb[tj][4] | (gb[tj][5] << 16),
                                  gb[tj][6] | (gb[tj][7] << 16)};
                b[tj] = __builtin_bit_cast(bf16x8, p);
            }
#pragma unroll
            for (int ti = 0; ti < S::TI; ++ti)
#pragma unroll
                for (int tj = 0; tj < S::TJ; ++tj)
                    acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ti], b[tj], acc[ti][tj], 0, 0, 0);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
#pragma unroll
                for (int ti = 0; ti < S::TI; ++ti)
#pragma unroll
                    for (int tj = 0; tj < S::TJ; ++tj)
                        acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[ti][e], gb[tj][e], acc[ti][tj], 0, 0, 0);
        }
    }

    // register v of lane (i, h) holds element (8 (v / 4) + 4 h + v % 4, i) of its 32x32 tile
    float *mine = partial + me * (int64_t)(FIN * FOUT);
#pragma unroll
    for (int ti = 0; ti < S::TI; ++ti)
#pragma unroll
        for (int tj = 0; tj < S::TJ; ++tj)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = (it0 + ti) * 32 + 8 * (v / 4) + 4 * hh + v % 4;
                const int c = (jt0 + tj) * 32 + i;
                if (r < FIN && c < FOUT) mine[r * FOUT + c] = acc[ti][tj][v];
            }
}

// dw[e] = (accumulate ? dw[e] : 0) + sum over the workers' partial results: sixteen wavefronts take a slice of
// the workers each (in worker order), then the sixteen slice sums are added in slice order: a fixed order.
constexpr int kReduceSlices = 16;
__global__ __launch_bounds__(kReduceSlices *kWave) void wgrad_reduce_kernel(const float *__restrict__ partial, int workers,
                                                                            int elems, float *__restrict__ dw,
                                                                            int accumulate) {
    __shared__ float s_sum[kReduceSlices][kWave];
    const int lane = threadIdx.x & (kWave - 1), slice = threadIdx.x / kWave;
    const int e = blockIdx.x * kWave + lane;
    const int per = (workers + kReduceSlices - 1) / kReduceSlices;
    const int p0 = slice * per, p1 = min(p0 + per, workers);
    float sum = 0.0f;
    if (e < elems) {
#pragma unroll 8
        for (int p = p0; p < p1; ++p) sum += partial[(int64_t)p * elems + e];
    }
    s_sum[slice][lane] = sum;
    __syncthreads();
    if (slice == 0 && e < elems) {
        float total = s_sum[0][lane];
#pragma unroll
        for (int k = 1; k < kReduceSlices; ++k) total += s_sum[k][lane];
        dw[e] = accumulate ? dw[e] + total : total;
    }
}

// out = (Z > 0 ? G : 0) * row_scale[row]; one 16-byte piece per lane.
template <bool BF16>
__global__ __launch_bounds__(kThreads) void relu_backward_kernel(const uintx4 *__restrict__ g, const uintx4 *__restrict__ z,
                                                                 const float *__restrict__ row_scale, uintx4 *__restrict__ out,
                                                                 int64_t pieces, int pieces_per_row) {
    const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p >= pieces) return;
    const uintx4 gv = __builtin_nontemporal_load(g + p), zv = __builtin_nontemporal_load(z + p);   // streams: read once
    const float sc = row_scale ? row_scale[p / pieces_per_row] : 1.0f;
    uintx4 o;
    if (BF16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            // a bf16 is positive when its sign bit is clear and it is not a zero
            const uint32_t zl = zv[e] & 0xffffu, zh = zv[e] >> 16;
            const float gl = __uint_as_float(gv[e] << 16), gh = __uint_as_float(gv[e] & 0xffff0000u);
            const float ol = (zl != 0u && zl < 0x8000u) ? gl * sc : 0.0f;
            const float oh = (zh != 0u && zh < 0x8000u) ? gh * sc : 0.0f;
            o[e] = f32_to_bf16(ol) | (f32_to_bf16(oh) << 16);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            o[e] = __float_as_uint(__uint_as_float(zv[e]) > 0.0f ? __uint_as_float(gv[e]) * sc : 0.0f);
    }
    __builtin_nontemporal_store(o, out + p);
}

template <int FIN, int FOUT, bool BF16>
int launch_wgrad(const void *x, const void *g, int64_t n, float *dw, int accumulate, float *partial, hipStream_t s) {
    using S = Split<FIN, FOUT>;
    const int64_t n_steps = (n + kStepRows - 1) / kStepRows;
    const int64_t needed = (n_steps + S::RS - 1) / S::RS;
    const int64_t blocks = std::min<int64_t>(std::min<int64_t>(needed, resident_workgroups(wgrad_kernel<FIN, FOUT, BF16>, kThreads, 512)), kMaxBlocks);
    hipLaunchKernelGGL((wgrad_kernel<FIN, FOUT, BF16>), dim3((unsigned)blocks), dim3(kThreads), 0, s, x, g, n, n_steps, partial);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    constexpr int elems = FIN * FOUT;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((elems + kWave - 1) / kWave), dim3(kReduceSlices * kWave), 0, s, partial,
                       (int)(blocks * S::RS), elems, dw, accumulate);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

template <int FIN, bool BF16>
int wgrad_out(int32_t f_out, const void *x, const void *g, int64_t n, float *dw, int accumulate, float *partial, hipStream_t s) {
    switch (f_out) {
        case 16: return launch_wgrad<FIN, 16, BF16>(x, g, n, dw, accumulate, partial, s);
        case 32: return launch_wgrad<FIN, 32, BF16>(x, g, n, dw, accumulate, partial, s);
        case 64: return launch_wgrad<FIN, 64, BF16>(x, g, n, dw, accumulate, partial, s);
        case 128: return launch_wgrad<FIN, 128, BF16>(x, g, n, dw, accumulate, partial, s);
        default: return DGNN_ERR_SHAPE;
    }
}

template <bool BF16>
int wgrad_in(int32_t f_in, int32_t f_out, const void *x, const void *g, int64_t n, float *dw, int accumulate, float *partial,
             hipStream_t s) {
    switch (f_in) {
        case 16: return wgrad_out<16, BF16>(f_out, x, g, n, dw, accumulate, partial, s);
        case 32: return wgrad_out<32, BF16>(f_out, x, g, n, dw, accumulate, partial, s);
        case 64: return wgrad_out<64, BF16>(f_out, x, g, n, dw, accumulate, partial, s);
        case 128: return wgrad_out<128, BF16>(f_out, x, g, n, dw, accumulate, partial, s);
        default: return DGNN_ERR_SHAPE;
    }
}

}  // namespace

extern "C" int dgnn_weight_grad_workspace(int32_t f_in, int32_t f_out, size_t *bytes) {
    if (!bytes) return DGNN_ERR_NULL;
    if (!supported_width(f_in) || !supported_width(f_out)) return DGNN_ERR_SHAPE;
    // one F x F' partial per row worker; a workgroup has at most four of them
    *bytes = (size_t)kMaxBlocks * kWavesPerBlock * (size_t)f_in * (size_t)f_out * sizeof(float);
    return DGNN_OK;
}

extern "C" int dgnn_weight_grad(const void *x, const void *g, int64_t n, int32_t f_in, int32_t f_out, float *dw,
                                int32_t accumulate, dgnn_dtype dt, void *ws, size_t ws_bytes, void *stream) {
    if (!x || !g || !dw || !ws) return DGNN_ERR_NULL;
    if (n <= 0 || !supported_width(f_in) || !supported_width(f_out)) return DGNN_ERR_SHAPE;
    if (dt != DGNN_F32 && dt != DGNN_BF16) return DGNN_ERR_SHAPE;
    if (!fits_index(n)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(x) || !aligned16(g) || !aligned16(ws)) return DGNN_ERR_ALIGN;
    size_t need = 0;
    dgnn_weight_grad_workspace(f_in, f_out, &need);
    if (ws_bytes < need) return DGNN_ERR_CAPACITY;
    hipStream_t s = (hipStream_t)stream;
    float *partial = static_cast<float *>(ws);
    return dt == DGNN_BF16 ? wgrad_in<true>(f_in, f_out, x, g, n, dw, accumulate ? 1 : 0, partial, s)
                           : wgrad_in<false>(f_in, f_out, x, g, n, dw, accumulate ? 1 : 0, partial, s);
}

extern "C" int dgnn_relu_backward(const void *g, const void *z, const float *row_scale, void *out, int64_t n, int32_t f,
                                  dgnn_dtype dt, void *stream) {
    if (!g || !z || !out) return DGNN_ERR_NULL;
    if (n <= 0 || !supported_width(f)) return DGNN_ERR_SHAPE;
    if (dt != DGNN_F32 && dt != DGNN_BF16) return DGNN_ERR_SHAPE;
    if (!fits_index(n)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(g) || !aligned16(z) || !aligned16(out)) return DGNN_ERR_ALIGN;
    const int pieces_per_row = f * (dt == DGNN_F32 ? 4 : 2) / 16;
    const int64_t pieces = n * pieces_per_row;
    const unsigned blocks = (unsigned)((pieces + kThreads - 1) / kThreads);
    hipStream_t s = (hipStream_t)stream;
    if (dt == DGNN_BF16)
        hipLaunchKernelGGL(relu_backward_kernel<true>, dim3(blocks), dim3(kThreads), 0, s, static_cast<const uintx4 *>(g),
                           static_cast<const uintx4 *>(z), row_scale, static_cast<uintx4 *>(out), pieces, pieces_per_row);
    else
        hipLaunchKernelGGL(relu_backward_kernel<false>, dim3(blocks), dim3(kThreads), 0, s, static_cast<const uintx4 *>(g),
                           static_cast<const uintx4 *>(z), row_scale, static_cast<uintx4 *>(out), pieces, pieces_per_row);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}
