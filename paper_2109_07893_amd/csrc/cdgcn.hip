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

constexpr int kThreads = 256;

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
    const uintx4 raw = __builtin_nontemporal_load(k < p0 ? y0 + row * p0 + k : y1 + row * p1 + (k - p0));   // streams
    float v[NV];
    Pack<BF16>::unpack(v, raw);
#pragma unroll
    for (int e = 0; e < NV; ++e) v[e] = fmaxf(v[e], 0.0f);
    __builtin_nontemporal_store(Pack<BF16>::pack(v), out + p);
}

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

// ---- One LSTM step with the gate pre-activations kept on chip -------------------------------------------
// a = [Y | h_prev] [W_x ; W_h] + b is 4 * hidden wide and, written out, is two thirds of the traffic of an LSTM
// step.  Here a wavefront takes 32 vertices, forms the TRANSPOSED gate tiles (W^T as the A operand, the rows
// of [Y | h_prev] as the B operand) on the matrix cores, and applies the cell straight to the accumulators.  Column
// C = g * hidden + k of the pre-activations is gate g of state element k; it lies in the 32-column tile C / 32, and
// lane (i, h) holds, for vertex i, the columns c of a tile with (c / 4) % 2 == h, four consecutive ones per four
// accumulator registers.  hidden is a multiple of 8, so the four gates of a state element sit in the same lane
// (hidden = 32: the four tiles ARE the four gates, same register slot in each).  Traffic: Y, h_prev, c in; c, h out.
// fp32 storage: hidden 16 or 32; bf16 storage (fp32 accumulation, the cell in fp32): hidden 32 or 64.
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// In the fused step the nonlinearities compete with the matrix cores for issue slots (they are as many cycles as
// the products when taken from the math library), so they are built from the hardware exponential and reciprocal:
// sig(x) = 1 / (1 + 2^(-x log2 e)), tanh(x) = 2 sig(2x) - 1; absolute error a few 1e-7.  The reciprocal is the
// hardware's approximation (1 ulp), one instruction where a correctly rounded one is a ten-instruction division.
__device__ __forceinline__ float fast_sigmoid(float x) { return __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }
__device__ __forceinline__ float fast_tanh(float x) { return 2.0f * fast_sigmoid(2.0f * x) - 1.0f; }

constexpr int kLstmHidden = 32;      // the bf16 adjoint kernel's only width
constexpr int kLstmThreads = 512;   // eight wavefronts share W in LDS: two per SIMD, so one multiplies while the other moves data
constexpr int kLstmWaves = kLstmThreads / kWave;

template <int FY, int HID>
__global__ __launch_bounds__(kLstmThreads) void lstm_step_f32_kernel(const float *__restrict__ y, const float *__restrict__ h_prev,
                                                                 const float *__restrict__ w_x, const float *__restrict__ w_h,
                                                                 const float *__restrict__ bias, float *c,
                                                                 float *__restrict__ h_next, int64_t n, int64_t n_tiles) {
    constexpr int G4 = 4 * HID, NT = G4 / 32;
    constexpr int K = FY + HID, KH = K / 2;
    constexpr int LDT = K + 4;                          // padded tile row (floats)
    constexpr int Y_PIECES = 32 * FY / 4 / kWave;       // 16-byte pieces per lane of a tile of Y
    constexpr int S_PIECES = 32 * HID / 4 / kWave;      // ... of a tile of h or c
    static_assert(K >= 2 * HID && KH % 4 == 0, "the tile buffer also carries c and h (2 * hidden columns)");
    // [W_x ; W_h] with the NT tiles' values of one (k, column-in-tile) side by side: s_w[(k * 32 + i) * NT + tile] is
    // element (k, tile * 32 + i), so one LDS read brings a k-step's operand for every tile
    __shared__ __attribute__((aligned(16))) float s_w[K * G4];
    __shared__ __attribute__((aligned(16))) float s_bias[G4];
    __shared__ __attribute__((aligned(16))) float s_tile[kLstmWaves][32 * LDT];

    const int tid = threadIdx.x;
    for (int idx = tid; idx < K * G4; idx += kLstmThreads) {
        const int k = idx / G4, col = idx % G4;
        s_w[(k * 32 + col % 32) * NT + col / 32] = idx < FY * G4 ? w_x[idx] : w_h[idx - FY * G4];
    }
    for (int idx = tid; idx < G4; idx += kLstmThreads) s_bias[idx] = bias ? bias[idx] : 0.0f;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int i = lane & 31, hh = lane >> 5;
    float *tile_lds = s_tile[wave];
    const int64_t stride = (int64_t)gridDim.x * kLstmWaves;
    const int64_t first = (int64_t)blockIdx.x * kLstmWaves + wave;
    __syncthreads();                                   // W is in LDS; from here on every wavefront is on its own
    // The rows of the next tile travel while this one is multiplied: a wavefront shares its SIMD with one other
    // only, which cannot hide a trip to memory per tile.
    const floatx4 zero = {0.f, 0.f, 0.f, 0.f};
    floatx4 yv[Y_PIECES], hv[S_PIECES], cv[S_PIECES];
    auto fetch = [&](int64_t t) {
#pragma unroll
        for (int q = 0; q < Y_PIECES; ++q) {
            const int64_t piece = t * (32 * FY / 4) + q * kWave + lane;
            yv[q] = (t < n_tiles && piece * 4 < n * FY) ? reinterpret_cast<const floatx4 *>(y)[piece] : zero;
        }
#pragma unroll
        for (int q = 0; q < S_PIECES; ++q) {
            const int64_t piece = t * (32 * HID / 4) + q * kWave + lane;
            const bool ok = t < n_tiles && piece * 4 < n * HID;
            hv[q] = ok ? reinterpret_cast<const floatx4 *>(h_prev)[piece] : zero;
            cv[q] = ok ? reinterpret_cast<const floatx4 *>(c)[piece] : zero;
        }
    };
    fetch(first);
    for (int64_t tile = first; tile < n_tiles; tile += stride) {
        // ---- [Y | h_prev] tile: registers -> LDS in whole lines
        floatx4 c_cur[S_PIECES];
#pragma unroll
        for (int q = 0; q < Y_PIECES; ++q) {
            const int e = (q * kWave + lane) * 4;
            *reinterpret_cast<floatx4 *>(&tile_lds[(e / FY) * LDT + e % FY]) = yv[q];
        }
#pragma unroll
        for (int q = 0; q < S_PIECES; ++q) {
            const int e = (q * kWave + lane) * 4;
            *reinterpret_cast<floatx4 *>(&tile_lds[(e / HID) * LDT + FY + e % HID]) = hv[q];
            c_cur[q] = cv[q];
        }
        fetch(tile + stride);          // another wavefront's tile: c is updated in place, but never a tile that is in flight
        wave_lds_sync();
        floatx4 a[KH / 4];
#pragma unroll
        for (int q = 0; q < KH / 4; ++q) a[q] = *reinterpret_cast<const floatx4 *>(&tile_lds[i * LDT + hh * KH + q * 4]);
        wave_lds_sync();                                                      // every lane has its operands
        // the tile buffer now takes the old cell state in columns [0, hidden)
#pragma unroll
        for (int q = 0; q < S_PIECES; ++q) {
            const int e = (q * kWave + lane) * 4;
            *reinterpret_cast<floatx4 *>(&tile_lds[(e / HID) * LDT + e % HID]) = c_cur[q];
        }
        floatx16 acc[NT];
#pragma unroll
        for (int g = 0; g < NT; ++g)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[g][v] = 0.0f;
#pragma unroll
        for (int s = 0; s < KH; ++s) {
            const float xv = a[s / 4][s % 4];
            float wv[NT];
#pragma unroll
            for (int g = 0; g < NT; ++g) wv[g] = s_w[((hh * KH + s) * 32 + i) * NT + g];   // consecutive: one read
#pragma unroll
            for (int g = 0; g < NT; ++g)
                acc[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(wv[g], xv, acc[g], 0, 0, 0);   // transposed tile g of the pre-activations
        }
        wave_lds_sync();                                                      // the old cell state is in LDS
        // ---- the cell, on the accumulators: lane (i, h) owns state elements 8 m + 4 h + r of vertex i; gate g of
        // them is column g * hidden + 8 m + 4 h + r: tile (g * hidden + 8 m) / 32, registers 4 q + r with q the
        // 8-column group inside the tile
#pragma unroll
        for (int m = 0; m < HID / 8; ++m) {
            const int k0 = 8 * m + 4 * hh;
            const floatx4 c_old = *reinterpret_cast<const floatx4 *>(&tile_lds[i * LDT + k0]);
            floatx4 c_new, h_new;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int k = k0 + r;
                const float ai = acc[(8 * m) / 32][4 * (((8 * m) % 32) / 8) + r] + s_bias[k];
                const float af = acc[(HID + 8 * m) / 32][4 * (((HID + 8 * m) % 32) / 8) + r] + s_bias[HID + k];
                const float ag = acc[(2 * HID + 8 * m) / 32][4 * (((2 * HID + 8 * m) % 32) / 8) + r] + s_bias[2 * HID + k];
                const float ao = acc[(3 * HID + 8 * m) / 32][4 * (((3 * HID + 8 * m) % 32) / 8) + r] + s_bias[3 * HID + k];
                c_new[r] = fast_sigmoid(af) * c_old[r] + fast_sigmoid(ai) * fast_tanh(ag);
                h_new[r] = fast_sigmoid(ao) * fast_tanh(c_new[r]);
            }
            *reinterpret_cast<floatx4 *>(&tile_lds[i * LDT + k0]) = c_new;
            *reinterpret_cast<floatx4 *>(&tile_lds[i * LDT + HID + k0]) = h_new;
        }
        wave_lds_sync();
        if (tile < n_tiles) {
#pragma unroll
            for (int q = 0; q < S_PIECES; ++q) {
                const int e = (q * kWave + lane) * 4;
                const int64_t piece = tile * (32 * HID / 4) + q * kWave + lane;
                if (piece * 4 < n * HID) {
                    reinterpret_cast<floatx4 *>(c)[piece] = *reinterpret_cast<const floatx4 *>(&tile_lds[(e / HID) * LDT + e % HID]);
                    reinterpret_cast<floatx4 *>(h_next)[piece] =
                        *reinterpret_cast<const floatx4 *>(&tile_lds[(e / HID) * LDT + HID + e % HID]);
                }
            }
        }
        wave_lds_sync();                                                      // the tile buffer is reused
    }
}

// The same step for bf16 storage: 16 k-values per matrix instruction (eight from each lane half), W^T parked in LDS
// with k contiguous, the tile buffer in bf16.  The cell runs in fp32 on the accumulators; c and h are rounded once,
// on the way out.  WAVES: wavefronts per workgroup (the widest case leaves room for four tile buffers beside W).
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <int FY, int HID, int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void lstm_step_bf16_kernel(const uint16_t *__restrict__ y, const uint16_t *__restrict__ h_prev,
                                                                      const uint16_t *__restrict__ w_x, const uint16_t *__restrict__ w_h,
                                                                      const float *__restrict__ bias, uint16_t *c,
                                                                      uint16_t *__restrict__ h_next, int64_t n, int64_t n_tiles) {
    constexpr int G4 = 4 * HID, NT = G4 / 32;
    constexpr int K = FY + HID, KH = K / 2, KS = KH / 8;
    constexpr int LDW = K + 8;                          // padded row of W^T (bf16 values)
    constexpr int LDT = K + 8;                          // padded tile row
    constexpr int Y_PIECES = 32 * FY / 8 / kWave;       // 16-byte pieces per lane of a tile of Y
    constexpr int S_PIECES = 32 * HID / 8 / kWave;      // ... of a tile of h or c
    static_assert(K >= 2 * HID && KH % 8 == 0, "the tile buffer also carries c and h (2 * hidden columns)");
    __shared__ __attribute__((aligned(16))) uint16_t s_wt[G4 * LDW];     // row j: column j of [W_x ; W_h]
    __shared__ __attribute__((aligned(16))) uint16_t s_tile[WAVES][32 * LDT];
    __shared__ __attribute__((aligned(16))) float s_bias[G4];

    const int tid = threadIdx.x;
    for (int idx = tid; idx < K * G4; idx += WAVES * kWave) {
        const int k = idx / G4, j = idx % G4;
        s_wt[j * LDW + k] = k < FY ? w_x[idx] : w_h[idx - FY * G4];
    }
    for (int idx = tid; idx < G4; idx += WAVES * kWave) s_bias[idx] = bias ? bias[idx] : 0.0f;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int i = lane & 31, hh = lane >> 5;
    uint16_t *tile_lds = s_tile[wave];
    const int64_t stride = (int64_t)gridDim.x * WAVES;
    const int64_t first = (int64_t)blockIdx.x * WAVES + wave;
    __syncthreads();                                   // W is in LDS; from here on every wavefront is on its own
    const uintx4 zero = {0u, 0u, 0u, 0u};
    uintx4 yv[Y_PIECES], hv[S_PIECES], cv[S_PIECES];        // the next tile's rows, fetched while this one is multiplied
    auto fetch = [&](int64_t t) {
#pragma unroll
        for (int q = 0; q < Y_PIECES; ++q) {
            const int64_t piece = t * (32 * FY / 8) + q * kWave + lane;
            yv[q] = (t < n_tiles && piece * 8 < n * FY) ? reinterpret_cast<const uintx4 *>(y)[piece] : zero;
        }
#pragma unroll
        for (int q = 0; q < S_PIECES; ++q) {
            const int64_t piece = t * (32 * HID / 8) + q * kWave + lane;
            const bool ok = t < n_tiles && piece * 8 < n * HID;
            hv[q] = ok ? reinterpret_cast<const uintx4 *>(h_prev)[piece] : zero;
            cv[q] = ok ? reinterpret_cast<const uintx4 *>(c)[piece] : zero;
        }
    };
    fetch(first);
    for (int64_t tile = first; tile < n_tiles; tile += stride) {
        uintx4 c_cur[S_PIECES];
#pragma unroll
        for (int q = 0; q < Y_PIECES; ++q) {
            const int e = (q * kWave + lane) * 8;
            *reinterpret_cast<uintx4 *>(&tile_lds[(e / FY) * LDT + e % FY]) = yv[q];
        }
#pragma unroll
        for (int q = 0; q < S_PIECES; ++q) {
            const int e = (q * kWave + lane) * 8;
            *reinterpret_cast<uintx4 *>(&tile_lds[(e / HID) * LDT + FY + e % HID]) = hv[q];
            c_cur[q] = cv[q];
        }
        fetch(tile + stride);
        wave_lds_sync();
        bf16x8 a[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) a[s] = *reinterpret_cast<const bf16x8 *>(&tile_lds[i * LDT + hh * KH + s * 8]);
        wave_lds_sync();                                                      // every lane has its operands
        // the tile buffer now takes the old cell state in columns [0, hidden)
#pragma unroll
        for (int q = 0; q < S_PIECES; ++q) {
            const int e = (q * kWave + lane) * 8;
            *reinterpret_cast<uintx4 *>(&tile_lds[(e / HID) * LDT + e % HID]) = c_cur[q];
        }
        floatx16 acc[NT];
#pragma unroll
        for (int g = 0; g < NT; ++g)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[g][v] = 0.0f;
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int g = 0; g < NT; ++g) {
                const bf16x8 wv = *reinterpret_cast<const bf16x8 *>(&s_wt[(g * 32 + i) * LDW + hh * KH + s * 8]);
                acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, a[s], acc[g], 0, 0, 0);    // transposed tile g of the pre-activations
            }
        wave_lds_sync();                                                      // the old cell state is in LDS
        // ---- the cell, on the accumulators (same ownership as in the fp32 kernel)
#pragma unroll
        for (int m = 0; m < HID / 8; ++m) {
            const int k0 = 8 * m + 4 * hh;
            const uint2 c_raw = *reinterpret_cast<const uint2 *>(&tile_lds[i * LDT + k0]);
            const float c_old[4] = {bf16_to_f32(c_raw.x & 0xffffu), bf16_to_f32(c_raw.x >> 16), bf16_to_f32(c_raw.y & 0xffffu),
                                    bf16_to_f32(c_raw.y >> 16)};
            float c_new[4], h_new[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int k = k0 + r;
                const float ai = acc[(8 * m) / 32][4 * (((8 * m) % 32) / 8) + r] + s_bias[k];
                const float af = acc[(HID + 8 * m) / 32][4 * (((HID + 8 * m) % 32) / 8) + r] + s_bias[HID + k];
                const float ag = acc[(2 * HID + 8 * m) / 32][4 * (((2 * HID + 8 * m) % 32) / 8) + r] + s_bias[2 * HID + k];
                const float ao = acc[(3 * HID + 8 * m) / 32][4 * (((3 * HID + 8 * m) % 32) / 8) + r] + s_bias[3 * HID + k];
                c_new[r] = fast_sigmoid(af) * c_old[r] + fast_sigmoid(ai) * fast_tanh(ag);
                h_new[r] = fast_sigmoid(ao) * fast_tanh(c_new[r]);
            }
            *reinterpret_cast<uint2 *>(&tile_lds[i * LDT + k0]) =
                make_uint2(f32_to_bf16(c_new[0]) | (f32_to_bf16(c_new[1]) << 16), f32_to_bf16(c_new[2]) | (f32_to_bf16(c_new[3]) << 16));
            *reinterpret_cast<uint2 *>(&tile_lds[i * LDT + HID + k0]) =
                make_uint2(f32_to_bf16(h_new[0]) | (f32_to_bf16(h_new[1]) << 16), f32_to_bf16(h_new[2]) | (f32_to_bf16(h_new[3]) << 16));
        }
        wave_lds_sync();
#pragma unroll
        for (int q = 0; q < S_PIECES; ++q) {
            const int e = (q * kWave + lane) * 8;
            const int64_t piece = tile * (32 * HID / 8) + q * kWave + lane;
            if (piece * 8 < n * HID) {
                reinterpret_cast<uintx4 *>(c)[piece] = *reinterpret_cast<const uintx4 *>(&tile_lds[(e / HID) * LDT + e % HID]);
                reinterpret_cast<uintx4 *>(h_next)[piece] = *reinterpret_cast<const uintx4 *>(&tile_lds[(e / HID) * LDT + HID + e % HID]);
            }
        }
        wave_lds_sync();                                                      // the tile buffer is reused
    }
}

// ---- The adjoint of that step, gate pre-activations recomputed on chip ----------------------------------------
// Same tiles, same products; the cell's backward formulas are applied to the accumulators instead:
//     dc = dh o (1 - tanh(c_t)^2) + dc_t,   da_i = dc g i (1 - i),  da_f = dc c_{t-1} f (1 - f),
//     da_g = dc i (1 - g^2),  da_o = dh tanh(c_t) o (1 - o),   dc_{t-1} = dc f.
// Traffic: Y, h_prev, c_prev, the incoming gradients in; da (4 * hidden wide) and dc_{t-1} out, instead of writing
// and re-reading both halves of the pre-activations as well.
template <int FY, int HID>
__global__ __launch_bounds__(kLstmThreads) void lstm_step_backward_f32_kernel(
    const float *__restrict__ y, const float *__restrict__ h_prev, const float *__restrict__ w_x, const float *__restrict__ w_h,
    const float *__restrict__ bias, const float *__restrict__ c_prev, const float *__restrict__ dh_a,
    const float *__restrict__ dh_b, const float *dc_next, float *__restrict__ da, float *dc_prev, int64_t n, int64_t n_tiles) {
    constexpr int G4 = 4 * HID, NT = G4 / 32;
    constexpr int K = FY + HID, KH = K / 2;
    constexpr int LDT = (K > 3 * HID ? K : 3 * HID) + 4;      // the tile buffer also carries c_prev, dh and dc side by side
    constexpr int Y_PIECES = 32 * FY / 4 / kWave;
    constexpr int S_PIECES = 32 * HID / 4 / kWave;
    constexpr int HALF_PIECES = 32 * (2 * HID) / 4 / kWave;   // 16-byte pieces per lane of half a tile of da
    static_assert(KH % 4 == 0, "operand rows are read in 16-byte pieces");
    __shared__ __attribute__((aligned(16))) float s_w[K * G4];      // laid out as in the forward kernel
    __shared__ __attribute__((aligned(16))) float s_bias[G4];
    __shared__ __attribute__((aligned(16))) float s_tile[kLstmWaves][32 * LDT];

    const int tid = threadIdx.x;
    for (int idx = tid; idx < K * G4; idx += kLstmThreads) {
        const int k = idx / G4, col = idx % G4;
        s_w[(k * 32 + col % 32) * NT + col / 32] = idx < FY * G4 ? w_x[idx] : w_h[idx - FY * G4];
    }
    for (int idx = tid; idx < G4; idx += kLstmThreads) s_bias[idx] = bias ? bias[idx] : 0.0f;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int i = lane & 31, hh = lane >> 5;
    float *tile_lds = s_tile[wave];
    const int64_t stride = (int64_t)gridDim.x * kLstmWaves;
    const int64_t first = (int64_t)blockIdx.x * kLstmWaves + wave;
    __syncthreads();
    for (int64_t tile = first; tile < n_tiles; tile += stride) {
        const floatx4 zero = {0.f, 0.f, 0.f, 0.f};
        floatx4 c_cur[S_PIECES], dh_cur[S_PIECES], dc_cur[S_PIECES];
        {
            floatx4 yv[Y_PIECES], hv[S_PIECES];
#pragma unroll
            for (int q = 0; q < Y_PIECES; ++q) {
                const int64_t piece = tile * (32 * FY / 4) + q * kWave + lane;
                yv[q] = piece * 4 < n * FY ? reinterpret_cast<const floatx4 *>(y)[piece] : zero;
            }
#pragma unroll
            for (int q = 0; q < S_PIECES; ++q) {
                const int64_t piece = tile * (32 * HID / 4) + q * kWave + lane;
                const bool ok = piece * 4 < n * HID;
                hv[q] = ok ? reinterpret_cast<const floatx4 *>(h_prev)[piece] : zero;
                c_cur[q] = ok ? reinterpret_cast<const floatx4 *>(c_prev)[piece] : zero;
                dh_cur[q] = (ok && dh_a) ? reinterpret_cast<const floatx4 *>(dh_a)[piece] : zero;
                if (ok && dh_b) dh_cur[q] += reinterpret_cast<const floatx4 *>(dh_b)[piece];
                dc_cur[q] = (ok && dc_next) ? reinterpret_cast<const floatx4 *>(dc_next)[piece] : zero;
            }
#pragma unroll
            for (int q = 0; q < Y_PIECES; ++q) {
                const int e = (q * kWave + lane) * 4;
                *reinterpret_cast<floatx4 *>(&tile_lds[(e / FY) * LDT + e % FY]) = yv[q];
            }
#pragma unroll
            for (int q = 0; q < S_PIECES; ++q) {
                const int e = (q * kWave + lane) * 4;
                *reinterpret_cast<floatx4 *>(&tile_lds[(e / HID) * LDT + FY + e % HID]) = hv[q];
            }
        }
        wave_lds_sync();
        floatx4 a[KH / 4];
#pragma unroll
        for (int q = 0; q < KH / 4; ++q) a[q] = *reinterpret_cast<const floatx4 *>(&tile_lds[i * LDT + hh * KH + q * 4]);
        wave_lds_sync();                                                      // every lane has its operands
        // the tile buffer now takes c_prev, dh and dc in columns [0, hidden), [hidden, 2 hidden), [2 hidden, 3 hidden)
#pragma unroll
        for (int q = 0; q < S_PIECES; ++q) {
            const int e = (q * kWave + lane) * 4;
            float *row = &tile_lds[(e / HID) * LDT + e % HID];
            *reinterpret_cast<floatx4 *>(row) = c_cur[q];
            *reinterpret_cast<floatx4 *>(row + HID) = dh_cur[q];
            *reinterpret_cast<floatx4 *>(row + 2 * HID) = dc_cur[q];
        }
        floatx16 acc[NT];
#pragma unroll
        for (int g = 0; g < NT; ++g)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[g][v] = 0.0f;
#pragma unroll
        for (int s = 0; s < KH; ++s) {
            const float xv = a[s / 4][s % 4];
            float wv[NT];
#pragma unroll
            for (int g = 0; g < NT; ++g) wv[g] = s_w[((hh * KH + s) * 32 + i) * NT + g];   // consecutive: one read
#pragma unroll
            for (int g = 0; g < NT; ++g) acc[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(wv[g], xv, acc[g], 0, 0, 0);   // transposed tile g of the pre-activations
        }
        wave_lds_sync();                                                      // c_prev, dh, dc are in LDS
        // ---- the cell's adjoint, on the accumulators: lane (i, h) owns state elements 8 m + 4 h + r of vertex i; gate g
        // of them is column g * hidden + 8 m + 4 h + r, in tile (g * hidden + 8 m) / 32, registers 4 q + r with q the
        // 8-column group inside the tile.  The gradients replace the pre-activations in the accumulators, dc_{t-1}
        // goes to the tile
#pragma unroll
        for (int m = 0; m < HID / 8; ++m) {
            const int k0 = 8 * m + 4 * hh;
            constexpr int kGroup = 8;
            const int ti = (0 * HID + kGroup * m) / 32, qi = ((0 * HID + kGroup * m) % 32) / 8;
            const int tf = (1 * HID + kGroup * m) / 32, qf = ((1 * HID + kGroup * m) % 32) / 8;
            const int tg = (2 * HID + kGroup * m) / 32, qg = ((2 * HID + kGroup * m) % 32) / 8;
            const int to = (3 * HID + kGroup * m) / 32, qo = ((3 * HID + kGroup * m) % 32) / 8;
            const floatx4 c_old = *reinterpret_cast<const floatx4 *>(&tile_lds[i * LDT + k0]);
            const floatx4 dh = *reinterpret_cast<const floatx4 *>(&tile_lds[i * LDT + HID + k0]);
            const floatx4 dc_in = *reinterpret_cast<const floatx4 *>(&tile_lds[i * LDT + 2 * HID + k0]);
            floatx4 dc_out;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int k = k0 + r;
                const float gi = fast_sigmoid(acc[ti][4 * qi + r] + s_bias[k]);
                const float gf = fast_sigmoid(acc[tf][4 * qf + r] + s_bias[HID + k]);
                const float gg = fast_tanh(acc[tg][4 * qg + r] + s_bias[2 * HID + k]);
                const float go = fast_sigmoid(acc[to][4 * qo + r] + s_bias[3 * HID + k]);
                const float tc = fast_tanh(gf * c_old[r] + gi * gg);
                const float d = dh[r] * go * (1.0f - tc * tc) + dc_in[r];
                acc[ti][4 * qi + r] = d * gg * gi * (1.0f - gi);
                acc[tf][4 * qf + r] = d * c_old[r] * gf * (1.0f - gf);
                acc[tg][4 * qg + r] = d * gi * (1.0f - gg * gg);
                acc[to][4 * qo + r] = dh[r] * tc * go * (1.0f - go);
                dc_out[r] = d * gf;
            }
            *reinterpret_cast<floatx4 *>(&tile_lds[i * LDT + k0]) = dc_out;          // over c_prev: this lane alone read it
        }
        wave_lds_sync();
#pragma unroll
        for (int q = 0; q < S_PIECES; ++q) {
            const int e = (q * kWave + lane) * 4;
            const int64_t piece = tile * (32 * HID / 4) + q * kWave + lane;
            if (piece * 4 < n * HID)
                reinterpret_cast<floatx4 *>(dc_prev)[piece] = *reinterpret_cast<const floatx4 *>(&tile_lds[(e / HID) * LDT + e % HID]);
        }
        // da leaves in two halves of two gates each (a whole tile of it does not fit the buffer): columns
        // [0, 2 hidden) of the tile rows, then whole stretches of 2 hidden values of da's rows
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            wave_lds_sync();                                                  // the buffer's previous contents have been read
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int m = 0; m < HID / 8; ++m) {
                    const int col = (2 * half + g) * HID + 8 * m;             // first column of the group in da's row
                    const floatx16 &src = acc[col / 32];
                    const int q = (col % 32) / 8;
                    *reinterpret_cast<floatx4 *>(&tile_lds[i * LDT + g * HID + 8 * m + 4 * hh]) =
                        floatx4{src[4 * q], src[4 * q + 1], src[4 * q + 2], src[4 * q + 3]};
                }
            wave_lds_sync();
#pragma unroll
            for (int q = 0; q < HALF_PIECES; ++q) {
                const int e = (q * kWave + lane) * 4;                          // element of the 32 x 64 half tile
                const int r = e / (2 * HID), col = e % (2 * HID);
                const int64_t row = tile * 32 + r;
                if (row < n)
                    *reinterpret_cast<floatx4 *>(&da[row * G4 + half * 2 * HID + col]) =
                        *reinterpret_cast<const floatx4 *>(&tile_lds[r * LDT + col]);
            }
        }
        wave_lds_sync();                                                      // the tile buffer is reused
    }
}

// The adjoint for bf16 storage, hidden = 32: products as in lstm_step_bf16_kernel, the cell's backward formulas in fp32
// on the accumulators; the two summands of dL/dh stay apart until they are added in fp32.
template <int FY>
__global__ __launch_bounds__(kLstmThreads) void lstm_step_backward_bf16_kernel(
    const uint16_t *__restrict__ y, const uint16_t *__restrict__ h_prev, const uint16_t *__restrict__ w_x,
    const uint16_t *__restrict__ w_h, const float *__restrict__ bias, const uint16_t *__restrict__ c_prev,
    const uint16_t *__restrict__ dh_a, const uint16_t *__restrict__ dh_b, const uint16_t *dc_next, uint16_t *__restrict__ da,
    uint16_t *dc_prev, int64_t n, int64_t n_tiles) {
    constexpr int HID = kLstmHidden, G4 = 4 * HID;
    constexpr int K = FY + HID, KH = K / 2, KS = KH / 8;
    constexpr int LDW = K + 8;
    constexpr int LDT = (K > 4 * HID ? K : 4 * HID) + 8;      // the tile buffer also carries c_prev, the two dh and dc side by side
    constexpr int Y_PIECES = 32 * FY / 8 / kWave;
    constexpr int S_PIECES = 32 * HID / 8 / kWave;
    constexpr int HALF_PIECES = 32 * (2 * HID) / 8 / kWave;   // 16-byte pieces per lane of half a tile of da
    static_assert(KH % 8 == 0, "operand rows are read in 16-byte pieces");
    __shared__ __attribute__((aligned(16))) uint16_t s_wt[G4 * LDW];
    __shared__ __attribute__((aligned(16))) float s_bias[G4];
    __shared__ __attribute__((aligned(16))) uint16_t s_tile[kLstmWaves][32 * LDT];

    const int tid = threadIdx.x;
    for (int idx = tid; idx < K * G4; idx += kLstmThreads) {
        const int k = idx / G4, j = idx % G4;
        s_wt[j * LDW + k] = k < FY ? w_x[idx] : w_h[idx - FY * G4];
    }
    for (int idx = tid; idx < G4; idx += kLstmThreads) s_bias[idx] = bias ? bias[idx] : 0.0f;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int i = lane & 31, hh = lane >> 5;
    uint16_t *tile_lds = s_tile[wave];
    const int64_t stride = (int64_t)gridDim.x * kLstmWaves;
    const int64_t first = (int64_t)blockIdx.x * kLstmWaves + wave;
    __syncthreads();
    auto unpack4 = [](uint2 r, float (&v)[4]) {
        v[0] = bf16_to_f32(r.x & 0xffffu); v[1] = bf16_to_f32(r.x >> 16);
        v[2] = bf16_to_f32(r.y & 0xffffu); v[3] = bf16_to_f32(r.y >> 16);
    };
    auto pack4 = [](const float (&v)[4]) {
        return make_uint2(f32_to_bf16(v[0]) | (f32_to_bf16(v[1]) << 16), f32_to_bf16(v[2]) | (f32_to_bf16(v[3]) << 16));
    };
    for (int64_t tile = first; tile < n_tiles; tile += stride) {
        const uintx4 zero = {0u, 0u, 0u, 0u};
        uintx4 c_cur[S_PIECES], dha_cur[S_PIECES], dhb_cur[S_PIECES], dc_cur[S_PIECES];
        {
            uintx4 yv[Y_PIECES], hv[S_PIECES];
#pragma unroll
            for (int q = 0; q < Y_PIECES; ++q) {
                const int64_t piece = tile * (32 * FY / 8) + q * kWave + lane;
                yv[q] = piece * 8 < n * FY ? reinterpret_cast<const uintx4 *>(y)[piece] : zero;
            }
#pragma unroll
            for (int q = 0; q < S_PIECES; ++q) {
                const int64_t piece = tile * (32 * HID / 8) + q * kWave + lane;
                const bool ok = piece * 8 < n * HID;
                hv[q] = ok ? reinterpret_cast<const uintx4 *>(h_prev)[piece] : zero;
                c_cur[q] = ok ? reinterpret_cast<const uintx4 *>(c_prev)[piece] : zero;
                dha_cur[q] = (ok && dh_a) ? reinterpret_cast<const uintx4 *>(dh_a)[piece] : zero;
                dhb_cur[q] = (ok && dh_b) ? reinterpret_cast<const uintx4 *>(dh_b)[piece] : zero;
                dc_cur[q] = (ok && dc_next) ? reinterpret_cast<const uintx4 *>(dc_next)[piece] : zero;
            }
#pragma unroll
            for (int q = 0; q < Y_PIECES; ++q) {
                const int e = (q * kWave + lane) * 8;
                *reinterpret_cast<uintx4 *>(&tile_lds[(e / FY) * LDT + e % FY]) = yv[q];
            }
#pragma unroll
            for (int q = 0; q < S_PIECES; ++q) {
                const int e = (q * kWave + lane) * 8;
                *reinterpret_cast<uintx4 *>(&tile_lds[(e / HID) * LDT + FY + e % HID]) = hv[q];
            }
        }
        wave_lds_sync();
        bf16x8 a[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) a[s] = *reinterpret_cast<const bf16x8 *>(&tile_lds[i * LDT + hh * KH + s * 8]);
        wave_lds_sync();                                                      // every lane has its operands
        // the tile buffer now takes c_prev, dh (two summands) and dc in four stretches of `hidden` columns
#pragma unroll
        for (int q = 0; q < S_PIECES; ++q) {
            const int e = (q * kWave + lane) * 8;
            uint16_t *row = &tile_lds[(e / HID) * LDT + e % HID];
            *reinterpret_cast<uintx4 *>(row) = c_cur[q];
            *reinterpret_cast<uintx4 *>(row + HID) = dha_cur[q];
            *reinterpret_cast<uintx4 *>(row + 2 * HID) = dhb_cur[q];
            *reinterpret_cast<uintx4 *>(row + 3 * HID) = dc_cur[q];
        }
        floatx16 acc[4];
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[g][v] = 0.0f;
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const bf16x8 wv = *reinterpret_cast<const bf16x8 *>(&s_wt[(g * 32 + i) * LDW + hh * KH + s * 8]);
                acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, a[s], acc[g], 0, 0, 0);    // transposed gate tile g
            }
        wave_lds_sync();                                                      // c_prev, dh, dc are in LDS
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int k0 = 8 * q + 4 * hh;
            float c_old[4], dha[4], dhb[4], dc_in[4], dc_out[4];
            unpack4(*reinterpret_cast<const uint2 *>(&tile_lds[i * LDT + k0]), c_old);
            unpack4(*reinterpret_cast<const uint2 *>(&tile_lds[i * LDT + HID + k0]), dha);
            unpack4(*reinterpret_cast<const uint2 *>(&tile_lds[i * LDT + 2 * HID + k0]), dhb);
            unpack4(*reinterpret_cast<const uint2 *>(&tile_lds[i * LDT + 3 * HID + k0]), dc_in);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int k = k0 + r;
                const float dh = dha[r] + dhb[r];
                const float gi = fast_sigmoid(acc[0][4 * q + r] + s_bias[k]);
                const float gf = fast_sigmoid(acc[1][4 * q + r] + s_bias[HID + k]);
                const float gg = fast_tanh(acc[2][4 * q + r] + s_bias[2 * HID + k]);
                const float go = fast_sigmoid(acc[3][4 * q + r] + s_bias[3 * HID + k]);
                const float tc = fast_tanh(gf * c_old[r] + gi * gg);
                const float d = dh * go * (1.0f - tc * tc) + dc_in[r];
                acc[0][4 * q + r] = d * gg * gi * (1.0f - gi);
                acc[1][4 * q + r] = d * c_old[r] * gf * (1.0f - gf);
                acc[2][4 * q + r] = d * gi * (1.0f - gg * gg);
                acc[3][4 * q + r] = dh * tc * go * (1.0f - go);
                dc_out[r] = d * gf;
            }
            *reinterpret_cast<uint2 *>(&tile_lds[i * LDT + k0]) = pack4(dc_out);         // over c_prev: this lane alone read it
        }
        wave_lds_sync();
#pragma unroll
        for (int q = 0; q < S_PIECES; ++q) {
            const int e = (q * kWave + lane) * 8;
            const int64_t piece = tile * (32 * HID / 8) + q * kWave + lane;
            if (piece * 8 < n * HID)
                reinterpret_cast<uintx4 *>(dc_prev)[piece] = *reinterpret_cast<const uintx4 *>(&tile_lds[(e / HID) * LDT + e % HID]);
        }
        // da leaves in two halves of two gates each, as in the fp32 kernel
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            wave_lds_sync();                                                  // the buffer's previous contents have been read
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const floatx16 &src = acc[2 * half + g];
                    const float v[4] = {src[4 * q], src[4 * q + 1], src[4 * q + 2], src[4 * q + 3]};
                    *reinterpret_cast<uint2 *>(&tile_lds[i * LDT + g * HID + 8 * q + 4 * hh]) = pack4(v);
                }
            wave_lds_sync();
#pragma unroll
            for (int q = 0; q < HALF_PIECES; ++q) {
                const int e = (q * kWave + lane) * 8;                          // element of the 32 x 64 half tile
                const int r = e / (2 * HID), col = e % (2 * HID);
                const int64_t row = tile * 32 + r;
                if (row < n)
                    *reinterpret_cast<uintx4 *>(&da[row * G4 + half * 2 * HID + col]) =
                        *reinterpret_cast<const uintx4 *>(&tile_lds[r * LDT + col]);
            }
        }
        wave_lds_sync();                                                      // the tile buffer is reused
    }
}

template <int FY, int HID>
int launch_lstm_step(const void *y, const void *h_prev, const void *w_x, const void *w_h, const float *bias, void *c,
                     void *h_next, int64_t n, hipStream_t s) {
    const int64_t n_tiles = (n + 31) / 32;
    const int64_t needed = (n_tiles + kLstmWaves - 1) / kLstmWaves;
    const int64_t resident = resident_workgroups(lstm_step_f32_kernel<FY, HID>, kLstmThreads, 256);
    const unsigned blocks = (unsigned)(needed < resident ? needed : resident);
    hipLaunchKernelGGL((lstm_step_f32_kernel<FY, HID>), dim3(blocks), dim3(kLstmThreads), 0, s, static_cast<const float *>(y),
                       static_cast<const float *>(h_prev), static_cast<const float *>(w_x), static_cast<const float *>(w_h),
                       bias, static_cast<float *>(c), static_cast<float *>(h_next), n, n_tiles);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

template <int FY, int HID, int WAVES>
int launch_lstm_step_bf16(const void *y, const void *h_prev, const void *w_x, const void *w_h, const float *bias, void *c,
                          void *h_next, int64_t n, hipStream_t s) {
    const int64_t n_tiles = (n + 31) / 32;
    const int64_t needed = (n_tiles + WAVES - 1) / WAVES;
    const int64_t resident = resident_workgroups(lstm_step_bf16_kernel<FY, HID, WAVES>, WAVES * kWave, 256);
    const unsigned blocks = (unsigned)(needed < resident ? needed : resident);
    hipLaunchKernelGGL((lstm_step_bf16_kernel<FY, HID, WAVES>), dim3(blocks), dim3(WAVES * kWave), 0, s, static_cast<const uint16_t *>(y),
                       static_cast<const uint16_t *>(h_prev), static_cast<const uint16_t *>(w_x), static_cast<const uint16_t *>(w_h),
                       bias, static_cast<uint16_t *>(c), static_cast<uint16_t *>(h_next), n, n_tiles);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

// The shapes the fused step is built for: hidden and, for each, the widths of Y (hidden and 2 * hidden: the layer's
// input is the concatenation of two blocks of features).
bool lstm_step_shape_ok(int32_t f_y, int32_t hidden, dgnn_dtype dt) {
    if (dt == DGNN_F32) return (hidden == 16 || hidden == 32) && (f_y == hidden || f_y == 2 * hidden);
    if (dt == DGNN_BF16) return (hidden == 32 || hidden == 64) && (f_y == hidden || f_y == 2 * hidden);
    return false;
}

}  // namespace

extern "C" int dgnn_lstm_step(const void *y, int32_t f_y, const void *h_prev, const void *w_x, const void *w_h,
                              const float *bias, void *c, void *h_next, int64_t n, int32_t hidden, dgnn_dtype dt,
                              void *stream) {
    if (!y || !h_prev || !w_x || !w_h || !c || !h_next) return DGNN_ERR_NULL;
    if (n <= 0 || !lstm_step_shape_ok(f_y, hidden, dt)) return DGNN_ERR_SHAPE;
    if (!fits_index(n)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(y) || !aligned16(h_prev) || !aligned16(c) || !aligned16(h_next)) return DGNN_ERR_ALIGN;
    if (h_next == h_prev || h_next == c || h_next == y || c == y || c == h_prev) return DGNN_ERR_ALIAS;
    hipStream_t s = (hipStream_t)stream;
    if (dt == DGNN_F32) {
        if (hidden == 32) return f_y == 32 ? launch_lstm_step<32, 32>(y, h_prev, w_x, w_h, bias, c, h_next, n, s)
                                           : launch_lstm_step<64, 32>(y, h_prev, w_x, w_h, bias, c, h_next, n, s);
        return f_y == 16 ? launch_lstm_step<16, 16>(y, h_prev, w_x, w_h, bias, c, h_next, n, s)
                         : launch_lstm_step<32, 16>(y, h_prev, w_x, w_h, bias, c, h_next, n, s);
    }
    if (hidden == 32) return f_y == 32 ? launch_lstm_step_bf16<32, 32, 8>(y, h_prev, w_x, w_h, bias, c, h_next, n, s)
                                       : launch_lstm_step_bf16<64, 32, 8>(y, h_prev, w_x, w_h, bias, c, h_next, n, s);
    return f_y == 64 ? launch_lstm_step_bf16<64, 64, 8>(y, h_prev, w_x, w_h, bias, c, h_next, n, s)
                     : launch_lstm_step_bf16<128, 64, 4>(y, h_prev, w_x, w_h, bias, c, h_next, n, s);
}

extern "C" int dgnn_lstm_step_backward(const void *y, int32_t f_y, const void *h_prev, const void *w_x, const void *w_h,
                                       const float *bias, const void *c_prev, const void *dh_a, const void *dh_b,
                                       const void *dc_next, void *da, void *dc_prev, int64_t n, int32_t hidden, dgnn_dtype dt,
                                       void *stream) {
    if (!y || !h_prev || !w_x || !w_h || !c_prev || !da || !dc_prev) return DGNN_ERR_NULL;
    if (!dh_a && !dh_b && !dc_next) return DGNN_ERR_NULL;
    if (n <= 0 || (dt != DGNN_F32 && dt != DGNN_BF16)) return DGNN_ERR_SHAPE;
    // fp32: hidden 16 or 32; bf16: hidden 32; Y as wide as the state or twice as wide
    if (!(hidden == 32 || (hidden == 16 && dt == DGNN_F32)) || (f_y != hidden && f_y != 2 * hidden)) return DGNN_ERR_SHAPE;
    if (!fits_index(n)) return DGNN_ERR_OVERFLOW;
    for (const void *p : {y, h_prev, c_prev, dh_a, dh_b, dc_next, (const void *)da, (const void *)dc_prev})
        if (p && !aligned16(p)) return DGNN_ERR_ALIGN;
    if (da == y || da == h_prev || da == c_prev || da == dh_a || da == dh_b || da == dc_next || da == dc_prev ||
        dc_prev == y || dc_prev == h_prev || dc_prev == c_prev || dc_prev == dh_a || dc_prev == dh_b)
        return DGNN_ERR_ALIAS;                                     // dc_prev may be dc_next: a tile is read before it is written
    const int64_t n_tiles = (n + 31) / 32;
    const int64_t needed = (n_tiles + kLstmWaves - 1) / kLstmWaves;
    auto launch = [&](auto kernel, auto elem) {
        typedef decltype(elem) E;
        const int64_t resident = resident_workgroups(kernel, kLstmThreads, 256);
        const unsigned blocks = (unsigned)(needed < resident ? needed : resident);
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(kLstmThreads), 0, (hipStream_t)stream, static_cast<const E *>(y),
                           static_cast<const E *>(h_prev), static_cast<const E *>(w_x), static_cast<const E *>(w_h),
                           bias, static_cast<const E *>(c_prev), static_cast<const E *>(dh_a),
                           static_cast<const E *>(dh_b), static_cast<const E *>(dc_next), static_cast<E *>(da),
                           static_cast<E *>(dc_prev), n, n_tiles);
    };
    if (dt == DGNN_F32) {
        if (hidden == 32) {
            if (f_y == 64) launch(lstm_step_backward_f32_kernel<64, 32>, float()); else launch(lstm_step_backward_f32_kernel<32, 32>, float());
        } else {
            if (f_y == 32) launch(lstm_step_backward_f32_kernel<32, 16>, float()); else launch(lstm_step_backward_f32_kernel<16, 16>, float());
        }
    } else {
        if (f_y == 64) launch(lstm_step_backward_bf16_kernel<64>, uint16_t()); else launch(lstm_step_backward_bf16_kernel<32>, uint16_t());
    }
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}
