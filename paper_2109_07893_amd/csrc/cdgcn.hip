// The two elementwise steps of the CD-GCN layer (Section "CD-GCN") that the shared kernels do not cover:
//   - the skip connection of its GCN operation, Y = sigma(Y0 o Y1) with Y0 = A~ X and Y1 = Y0 W laid side by
//     side (F + F' features per vertex);
//   - the cell of the LSTM that aggregates over time, state (h, c) per vertex: with the four gate
//     pre-activations a = X_t W_x + h_{t-1} W_h + b split as (i, f, g, o),
//         c_t = sig(f) * c_{t-1} + sig(i) * tanh(g),    h_t = sig(o) * tanh(c_t).
// The two products that make the gate pre-activations are the dense transform; only their sum, the
// nonlinearities and the state update happen here.  Both kernels stream 16-byte pieces (HBM-bound).
#include "common.hpp"

namespace {

using namespace dgnn;

typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;

template <bool BF16> struct Pack;
template <> struct Pack<false> {
    static constexpr int kVals = 4;
    static __device__ __forceinline__ void unpack(float (&v)[4], uintx4 t) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = __uint_as_float(t[e]);
    }
    static __device__ __forceinline__ uintx4 pack(const float (&v)[4]) {
        return uintx4{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
    }
};
template <> struct Pack<true> {
    static constexpr int kVals = 8;
    static __device__ __forceinline__ void unpack(float (&v)[8], uintx4 t) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[2 * e] = __uint_as_float(t[e] << 16);
            v[2 * e + 1] = __uint_as_float(t[e] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ uintx4 pack(const float (&v)[8]) {
        uintx4 t;
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] = f32_to_bf16(v[2 * e]) | (f32_to_bf16(v[2 * e + 1]) << 16);
        return t;
    }
};

// out[r] = relu(y0[r] o y1[r]); p0, p1 = 16-byte pieces per row of y0, y1.
template <bool BF16>
__global__ __launch_bounds__(kThreads) void concat_relu_kernel(const uintx4 *__restrict__ y0, int p0,
                                                               const uintx4 *__restrict__ y1, int p1,
                                                               uintx4 *__restrict__ out, int64_t pieces) {
    constexpr int NV = Pack<BF16>::kVals;
    const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p >= pieces) return;
    const int64_t row = p / (p0 + p1);
    const int k = (int)(p - row * (p0 + p1));
    const uintx4 raw = k < p0 ? y0[row * p0 + k] : y1[row * p1 + (k - p0)];
    float v[NV];
    Pack<BF16>::unpack(v, raw);
#pragma unroll
    for (int e = 0; e < NV; ++e) v[e] = fmaxf(v[e], 0.0f);
    out[p] = Pack<BF16>::pack(v);
}

__device__ __forceinline__ float sigmoidf(float x) { return 1.0f / (1.0f + expf(-x)); }

// One 16-byte piece of the state per lane; the four gates of that piece lie `hp` pieces apart in a row of gates.
template <bool BF16>
__global__ __launch_bounds__(kThreads) void lstm_cell_kernel(const uintx4 *__restrict__ gx, const uintx4 *__restrict__ gh,
                                                             const float *__restrict__ bias, const uintx4 *c_prev,
                                                             uintx4 *c_next, uintx4 *__restrict__ h_next, int64_t pieces,
                                                             int hp) {
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
    float c[NV], hn[NV];
    Pack<BF16>::unpack(c, c_prev[p]);
#pragma unroll
    for (int e = 0; e < NV; ++e) {
        c[e] = sigmoidf(a[1][e]) * c[e] + sigmoidf(a[0][e]) * tanhf(a[2][e]);
        hn[e] = sigmoidf(a[3][e]) * tanhf(c[e]);
    }
    c_next[p] = Pack<BF16>::pack(c);
    h_next[p] = Pack<BF16>::pack(hn);
}

}  // namespace

extern "C" int dgnn_concat_relu(const void *y0, int32_t f0, const void *y1, int32_t f1, void *out, int64_t n,
                                dgnn_dtype dt, void *stream) {
    if (!y0 || !y1 || !out) return DGNN_ERR_NULL;
    if (n <= 0 || !supported_width(f0) || !supported_width(f1)) return DGNN_ERR_SHAPE;
    if (dt != DGNN_F32 && dt != DGNN_BF16) return DGNN_ERR_SHAPE;
    if (!fits_index(n)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(y0) || !aligned16(y1) || !aligned16(out)) return DGNN_ERR_ALIGN;
    if (out == y0 || out == y1) return DGNN_ERR_ALIAS;
    const int s = dt == DGNN_F32 ? 4 : 2;
    const int p0 = f0 * s / 16, p1 = f1 * s / 16;
    const int64_t pieces = n * (p0 + p1);
    const unsigned blocks = (unsigned)((pieces + kThreads - 1) / kThreads);
    hipStream_t st = (hipStream_t)stream;
    if (dt == DGNN_BF16)
        hipLaunchKernelGGL(concat_relu_kernel<true>, dim3(blocks), dim3(kThreads), 0, st, static_cast<const uintx4 *>(y0), p0,
                           static_cast<const uintx4 *>(y1), p1, static_cast<uintx4 *>(out), pieces);
    else
        hipLaunchKernelGGL(concat_relu_kernel<false>, dim3(blocks), dim3(kThreads), 0, st, static_cast<const uintx4 *>(y0), p0,
                           static_cast<const uintx4 *>(y1), p1, static_cast<uintx4 *>(out), pieces);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

extern "C" int dgnn_lstm_cell(const void *gates_x, const void *gates_h, const float *bias, const void *c_prev, void *c_next,
                              void *h_next, int64_t n, int32_t hidden, dgnn_dtype dt, void *stream) {
    if (!gates_x || !gates_h || !c_prev || !c_next || !h_next) return DGNN_ERR_NULL;
    if (n <= 0 || !supported_width(hidden)) return DGNN_ERR_SHAPE;
    if (dt != DGNN_F32 && dt != DGNN_BF16) return DGNN_ERR_SHAPE;
    if (!fits_index(n)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(gates_x) || !aligned16(gates_h) || !aligned16(c_prev) || !aligned16(c_next) || !aligned16(h_next))
        return DGNN_ERR_ALIGN;
    if (h_next == gates_x || h_next == gates_h || h_next == c_prev || h_next == c_next || c_next == gates_x ||
        c_next == gates_h)
        return DGNN_ERR_ALIAS;
    const int hp = hidden * (dt == DGNN_F32 ? 4 : 2) / 16;
    const int64_t pieces = n * hp;
    const unsigned blocks = (unsigned)((pieces + kThreads - 1) / kThreads);
    hipStream_t st = (hipStream_t)stream;
    if (dt == DGNN_BF16)
        hipLaunchKernelGGL(lstm_cell_kernel<true>, dim3(blocks), dim3(kThreads), 0, st, static_cast<const uintx4 *>(gates_x),
                           static_cast<const uintx4 *>(gates_h), bias, static_cast<const uintx4 *>(c_prev),
                           static_cast<uintx4 *>(c_next), static_cast<uintx4 *>(h_next), pieces, hp);
    else
        hipLaunchKernelGGL(lstm_cell_kernel<false>, dim3(blocks), dim3(kThreads), 0, st, static_cast<const uintx4 *>(gates_x),
                           static_cast<const uintx4 *>(gates_h), bias, static_cast<const uintx4 *>(c_prev),
                           static_cast<uintx4 *>(c_next), static_cast<uintx4 *>(h_next), pieces, hp);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}
