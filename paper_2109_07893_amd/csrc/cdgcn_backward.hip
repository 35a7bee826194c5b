// Gradient propagation through the elementwise steps of the CD-GCN layer (Section "CD-GCN", trained as in
// Section "Gradient Checkpoint": the forward values are recomputed, not stored):
//   - the LSTM cell: from dL/dh_t, dL/dc_t and the recomputed gate pre-activations to dL/d(pre-activations)
//     and dL/dc_{t-1}.  With (i, f, g, o) = (sig, sig, tanh, sig) of the four pre-activations,
//     c_t = f c_{t-1} + i g and h_t = o tanh(c_t):
//         dc   = dh o (1 - tanh(c_t)^2) + dc_t
//         da_i = dc g i (1 - i),  da_f = dc c_{t-1} f (1 - f),  da_g = dc i (1 - g^2),  da_o = dh tanh(c_t) o (1 - o)
//         dc_{t-1} = dc f
//     everything else (dW_x, dW_h, dY, dh_{t-1}) is the dense transform's adjoints applied to da;
//   - the skip connection Y = relu(Y0 o Y1): dY masked by Y > 0 and split back into its two column blocks;
//   - the bias: column sums of da.
// All three stream 16-byte pieces (HBM-bound).
#include <algorithm>
#include <initializer_list>

#include "common.hpp"

namespace {

using namespace dgnn;

constexpr int kThreads = 256;
constexpr int kSumBlocks = 1024;       // workgroups (and partial sums per column) of the column-sum kernel

// One 16-byte piece of the state per lane; the four gates of that piece lie `hp` pieces apart in a row of gates.
template <bool BF16>
__global__ __launch_bounds__(kThreads) void lstm_cell_backward_kernel(
    const uintx4 *__restrict__ gx, const uintx4 *__restrict__ gh, const float *__restrict__ bias,
    const uintx4 *__restrict__ c_prev, const uintx4 *__restrict__ dh_a, const uintx4 *__restrict__ dh_b,
    const uintx4 *dc_next, uintx4 *__restrict__ da, uintx4 *dc_prev, int64_t pieces, int hp) {
    constexpr int NV = Pack<BF16>::kVals;
    const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p >= pieces) return;
    const int64_t row = p / hp;
    const int k = (int)(p - row * hp);
    float a[4][NV];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        float x[NV], h[NV];
        Pack<BF16>::unpack(x, gx[row * 4 * hp + q * hp + k]);
        Pack<BF16>::unpack(h, gh[row * 4 * hp + q * hp + k]);
#pragma unroll
        for (int e = 0; e < NV; ++e) a[q][e] = x[e] + h[e] + (bias ? bias[(q * hp + k) * NV + e] : 0.0f);
    }
    float c[NV], dh[NV], dc[NV], t[NV];
    Pack<BF16>::unpack(c, c_prev[p]);
#pragma unroll
    for (int e = 0; e < NV; ++e) dh[e] = dc[e] = 0.0f;
    if (dh_a) { Pack<BF16>::unpack(t, dh_a[p]);
#pragma unroll
        for (int e = 0; e < NV; ++e) dh[e] += t[e]; }
    if (dh_b) { Pack<BF16>::unpack(t, dh_b[p]);
#pragma unroll
        for (int e = 0; e < NV; ++e) dh[e] += t[e]; }
    if (dc_next) Pack<BF16>::unpack(dc, dc_next[p]);
    float out[4][NV], dcp[NV];
#pragma unroll
    for (int e = 0; e < NV; ++e) {
        const float i = sigmoidf(a[0][e]), f = sigmoidf(a[1][e]), g = tanhf(a[2][e]), o = sigmoidf(a[3][e]);
        const float tc = tanhf(f * c[e] + i * g);
        const float d = dh[e] * o * (1.0f - tc * tc) + dc[e];
        out[0][e] = d * g * i * (1.0f - i);
        out[1][e] = d * c[e] * f * (1.0f - f);
        out[2][e] = d * i * (1.0f - g * g);
        out[3][e] = dh[e] * tc * o * (1.0f - o);
        dcp[e] = d * f;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) da[row * 4 * hp + q * hp + k] = Pack<BF16>::pack(out[q]);
    dc_prev[p] = Pack<BF16>::pack(dcp);
}

// d0[r] o d1[r] = dy[r] where y[r] > 0, else 0; p0, p1 = 16-byte pieces per row of d0, d1 (d0 may be null).
template <bool BF16>
__global__ __launch_bounds__(kThreads) void concat_relu_backward_kernel(const uintx4 *__restrict__ dy,
                                                                        const uintx4 *__restrict__ y, uintx4 *__restrict__ d0,
                                                                        int p0, uintx4 *__restrict__ d1, int p1, int64_t pieces) {
    constexpr int NV = Pack<BF16>::kVals;
    const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p >= pieces) return;
    const int64_t row = p / (p0 + p1);
    const int k = (int)(p - row * (p0 + p1));
    if (k < p0 && !d0) return;
    float g[NV], v[NV];
    Pack<BF16>::unpack(g, dy[p]);
    Pack<BF16>::unpack(v, y[p]);
#pragma unroll
    for (int e = 0; e < NV; ++e) g[e] = v[e] > 0.0f ? g[e] : 0.0f;
    if (k < p0) d0[row * p0 + k] = Pack<BF16>::pack(g);
    else d1[row * p1 + (k - p0)] = Pack<BF16>::pack(g);
}

// Column sums, first stage: workgroup b adds the rows b, b + gridDim, ... (in that order, per column) and leaves
// one partial sum per column.  ppr = 16-byte pieces per row; a thread keeps one piece's columns.
template <bool BF16>
__global__ __launch_bounds__(kThreads) void column_sum_kernel(const uintx4 *__restrict__ g, int64_t n, int ppr,
                                                              float *__restrict__ partial) {
    constexpr int NV = Pack<BF16>::kVals;
    __shared__ float s_acc[kThreads * NV];
    const int rows_per_step = kThreads / ppr;            // ppr divides kThreads (widths are powers of two up to 128)
    const int k = threadIdx.x % ppr, sub = threadIdx.x / ppr;
    float acc[NV];
#pragma unroll
    for (int e = 0; e < NV; ++e) acc[e] = 0.0f;
    for (int64_t r = (int64_t)blockIdx.x * rows_per_step + sub; r < n; r += (int64_t)gridDim.x * rows_per_step) {
        float v[NV];
        Pack<BF16>::unpack(v, g[r * ppr + k]);
#pragma unroll
        for (int e = 0; e < NV; ++e) acc[e] += v[e];
    }
#pragma unroll
    for (int e = 0; e < NV; ++e) s_acc[threadIdx.x * NV + e] = acc[e];
    __syncthreads();
    if (sub == 0) {                                      // the threads of the first row add up their column's pieces in order
        for (int s = 1; s < rows_per_step; ++s)
#pragma unroll
            for (int e = 0; e < NV; ++e) acc[e] += s_acc[(s * ppr + k) * NV + e];
#pragma unroll
        for (int e = 0; e < NV; ++e) partial[(int64_t)blockIdx.x * ppr * NV + k * NV + e] = acc[e];
    }
}

// out = a + b, piece by piece (a gradient that reaches a tensor along two paths)
template <bool BF16>
__global__ __launch_bounds__(kThreads) void add_kernel(const uintx4 *a, const uintx4 *b, uintx4 *out, int64_t pieces) {
    constexpr int NV = Pack<BF16>::kVals;
    const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p >= pieces) return;
    float x[NV], y[NV];
    Pack<BF16>::unpack(x, a[p]);
    Pack<BF16>::unpack(y, b[p]);
#pragma unroll
    for (int e = 0; e < NV; ++e) x[e] += y[e];
    out[p] = Pack<BF16>::pack(x);
}

// second stage: db[c] (+)= sum over workgroups, in workgroup order
__global__ __launch_bounds__(kThreads) void column_sum_reduce_kernel(const float *__restrict__ partial, int blocks, int f,
                                                                     float *__restrict__ db, int accumulate) {
    const int c = blockIdx.x * kThreads + threadIdx.x;
    if (c >= f) return;
    float s = 0.0f;
    int b = 0;
    for (; b + 16 <= blocks; b += 16) {                  // sixteen loads in flight, added in workgroup order
        float v[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) v[q] = partial[(int64_t)(b + q) * f + c];
#pragma unroll
        for (int q = 0; q < 16; ++q) s += v[q];
    }
    for (; b < blocks; ++b) s += partial[(int64_t)b * f + c];
    db[c] = accumulate ? db[c] + s : s;
}

}  // namespace

extern "C" int dgnn_lstm_cell_backward(const void *gates_x, const void *gates_h, const float *bias, const void *c_prev,
                                       const void *dh_a, const void *dh_b, const void *dc_next, void *da, void *dc_prev,
                                       int64_t n, int32_t hidden, dgnn_dtype dt, void *stream) {
    if (!gates_x || !gates_h || !c_prev || !da || !dc_prev) return DGNN_ERR_NULL;
    if (!dh_a && !dh_b && !dc_next) return DGNN_ERR_NULL;            // no gradient arrives at all
    if (n <= 0 || !supported_width(hidden)) return DGNN_ERR_SHAPE;
    if (dt != DGNN_F32 && dt != DGNN_BF16) return DGNN_ERR_SHAPE;
    if (!fits_index(n)) return DGNN_ERR_OVERFLOW;
    for (const void *p : {gates_x, gates_h, c_prev, dh_a, dh_b, dc_next, (const void *)da, (const void *)dc_prev})
        if (p && !aligned16(p)) return DGNN_ERR_ALIGN;
    if (da == gates_x || da == gates_h || da == c_prev || da == dh_a || da == dh_b || da == dc_next || da == dc_prev ||
        dc_prev == gates_x || dc_prev == gates_h || dc_prev == c_prev || dc_prev == dh_a || dc_prev == dh_b)
        return DGNN_ERR_ALIAS;                                         // dc_prev may be dc_next: each lane reads its piece first
    const int hp = hidden * (dt == DGNN_F32 ? 4 : 2) / 16;
    const int64_t pieces = n * hp;
    const unsigned blocks = (unsigned)((pieces + kThreads - 1) / kThreads);
    hipStream_t st = (hipStream_t)stream;
    auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(kThreads), 0, st, static_cast<const uintx4 *>(gates_x),
                           static_cast<const uintx4 *>(gates_h), bias, static_cast<const uintx4 *>(c_prev),
                           static_cast<const uintx4 *>(dh_a), static_cast<const uintx4 *>(dh_b),
                           static_cast<const uintx4 *>(dc_next), static_cast<uintx4 *>(da), static_cast<uintx4 *>(dc_prev),
                           pieces, hp);
    };
    if (dt == DGNN_BF16) launch(lstm_cell_backward_kernel<true>); else launch(lstm_cell_backward_kernel<false>);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

extern "C" int dgnn_concat_relu_backward(const void *dy, const void *y, void *d0, int32_t f0, void *d1, int32_t f1, int64_t n,
                                         dgnn_dtype dt, void *stream) {
    if (!dy || !y || !d1) return DGNN_ERR_NULL;
    if (n <= 0 || !supported_width(f0) || !supported_width(f1)) return DGNN_ERR_SHAPE;
    if (dt != DGNN_F32 && dt != DGNN_BF16) return DGNN_ERR_SHAPE;
    if (!fits_index(n)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(dy) || !aligned16(y) || !aligned16(d1) || (d0 && !aligned16(d0))) return DGNN_ERR_ALIGN;
    if (d1 == dy || d1 == y || d0 == dy || d0 == y || d0 == d1) return DGNN_ERR_ALIAS;
    const int s = dt == DGNN_F32 ? 4 : 2;
    const int p0 = f0 * s / 16, p1 = f1 * s / 16;
    const int64_t pieces = n * (p0 + p1);
    const unsigned blocks = (unsigned)((pieces + kThreads - 1) / kThreads);
    hipStream_t st = (hipStream_t)stream;
    auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(kThreads), 0, st, static_cast<const uintx4 *>(dy),
                           static_cast<const uintx4 *>(y), static_cast<uintx4 *>(d0), p0, static_cast<uintx4 *>(d1), p1, pieces);
    };
    if (dt == DGNN_BF16) launch(concat_relu_backward_kernel<true>); else launch(concat_relu_backward_kernel<false>);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

extern "C" int dgnn_bias_grad_workspace(int32_t f, size_t *bytes) {
    if (!bytes) return DGNN_ERR_NULL;
    if (f <= 0 || f % 8 != 0 || f > 512) return DGNN_ERR_SHAPE;
    *bytes = (size_t)kSumBlocks * f * sizeof(float);
    return DGNN_OK;
}

extern "C" int dgnn_bias_grad(const void *g, int64_t n, int32_t f, float *db, int accumulate, dgnn_dtype dt, void *ws,
                              size_t ws_bytes, void *stream) {
    if (!g || !db || !ws) return DGNN_ERR_NULL;
    if (dt != DGNN_F32 && dt != DGNN_BF16) return DGNN_ERR_SHAPE;
    const int ppr = f * (dt == DGNN_F32 ? 4 : 2) / 16;
    // rows of 16-byte pieces whose count divides the workgroup: widths 4 * 2^k (fp32) / 8 * 2^k (bf16) up to 512
    if (n <= 0 || f <= 0 || f > 512 || ppr < 1 || ppr * 16 != f * (dt == DGNN_F32 ? 4 : 2) || (ppr & (ppr - 1)) || ppr > kThreads)
        return DGNN_ERR_SHAPE;
    if (!fits_index(n)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(g) || !aligned16(ws)) return DGNN_ERR_ALIGN;
    if (ws_bytes < (size_t)kSumBlocks * f * sizeof(float)) return DGNN_ERR_CAPACITY;
    hipStream_t st = (hipStream_t)stream;
    const int rows_per_step = kThreads / ppr;
    const int blocks = (int)std::min<int64_t>(kSumBlocks, (n + rows_per_step - 1) / rows_per_step);
    if (dt == DGNN_BF16)
        hipLaunchKernelGGL(column_sum_kernel<true>, dim3(blocks), dim3(kThreads), 0, st, static_cast<const uintx4 *>(g), n, ppr,
                           (float *)ws);
    else
        hipLaunchKernelGGL(column_sum_kernel<false>, dim3(blocks), dim3(kThreads), 0, st, static_cast<const uintx4 *>(g), n, ppr,
                           (float *)ws);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    hipLaunchKernelGGL(column_sum_reduce_kernel, dim3((f + kThreads - 1) / kThreads), dim3(kThreads), 0, st, (const float *)ws,
                       blocks, f, db, accumulate);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

extern "C" int dgnn_add(const void *a, const void *b, void *out, int64_t n, int32_t f, dgnn_dtype dt, void *stream) {
    if (!a || !b || !out) return DGNN_ERR_NULL;
    if (n <= 0 || !supported_width(f)) return DGNN_ERR_SHAPE;
    if (dt != DGNN_F32 && dt != DGNN_BF16) return DGNN_ERR_SHAPE;
    if (!fits_index(n)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(a) || !aligned16(b) || !aligned16(out)) return DGNN_ERR_ALIGN;
    const int64_t pieces = n * (f * (dt == DGNN_F32 ? 4 : 2) / 16);
    const unsigned blocks = (unsigned)((pieces + kThreads - 1) / kThreads);
    hipStream_t st = (hipStream_t)stream;
    if (dt == DGNN_BF16)
        hipLaunchKernelGGL(add_kernel<true>, dim3(blocks), dim3(kThreads), 0, st, static_cast<const uintx4 *>(a),
                           static_cast<const uintx4 *>(b), static_cast<uintx4 *>(out), pieces);
    else
        hipLaunchKernelGGL(add_kernel<false>, dim3(blocks), dim3(kThreads), 0, st, static_cast<const uintx4 *>(a),
                           static_cast<const uintx4 *>(b), static_cast<uintx4 *>(out), pieces);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}
