// M-transform of TM-GCN (Section "TM-GCN"): Y = Z x_1 M with the banded lower-triangular M,
//     Y_t = sum_{j=0}^{min(w,t)-1} m(t,j) Z_{t-j},   m(t,j) = 1/min(w,t) unless given.
//
// Each lane owns one 16-byte piece of the N x F frame and walks the time axis once, keeping the
// last w frames of its piece in a register ring, so every frame is read once and written once
// (2 s N F bytes per timestep) whatever the window, and the transform can run in place.
// The time loop is unrolled by the ring size so that ring slots are compile-time registers.
// With the paper's weights (every term 1/min(w,t)) the window sum is kept as a running sum,
// S_t = S_{t-1} + Z_t - Z_{t-w}, with a ring of exactly w slots (the slot about to be overwritten
// holds Z_{t-w}) and up to four frames fetched ahead; explicit coefficients take the general
// kernel, w multiply-adds per element.
#include "common.hpp"

namespace {

using namespace dgnn;

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;

template <bool BF16> struct Vec;
template <> struct Vec<false> {
    static constexpr int kVals = 4;
    static __device__ __forceinline__ void load(float (&v)[4], const char *p) {
        floatx4 t = *reinterpret_cast<const floatx4 *>(p);
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = t[e];
    }
    static __device__ __forceinline__ void store(char *p, const float (&v)[4]) {
        *reinterpret_cast<floatx4 *>(p) = floatx4{v[0], v[1], v[2], v[3]};
    }
    static __device__ __forceinline__ void unpack(float (&v)[4], uintx4 t) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = __uint_as_float(t[e]);
    }
};
template <> struct Vec<true> {
    static constexpr int kVals = 8;
    static __device__ __forceinline__ void load(float (&v)[8], const char *p) {
        uintx4 t = *reinterpret_cast<const uintx4 *>(p);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[2 * e] = __uint_as_float(t[e] << 16);
            v[2 * e + 1] = __uint_as_float(t[e] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ void store(char *p, const float (&v)[8]) {
        uintx4 t;
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] = f32_to_bf16(v[2 * e]) | (f32_to_bf16(v[2 * e + 1]) << 16);
        *reinterpret_cast<uintx4 *>(p) = t;
    }
    static __device__ __forceinline__ void unpack(float (&v)[8], uintx4 t) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[2 * e] = __uint_as_float(t[e] << 16);
            v[2 * e + 1] = __uint_as_float(t[e] & 0xffff0000u);
        }
    }
};

// RING >= w.  frame_bytes = n * f * s; pieces = frame_bytes / 16.
// REVERSE runs the adjoint, out_k = sum_j m(k + j, j) in_{k+j}: the same walk with the time axis turned round
// (step i handles frame T - 1 - i, the ring then holds the frames after it).
template <int RING, bool BF16, bool REVERSE>
__global__ __launch_bounds__(kThreads) void mproduct_kernel(const char *z, char *y, int T, int64_t pieces,
                                                            int64_t frame_bytes, int w, const float *__restrict__ m_band) {
    constexpr int NV = Vec<BF16>::kVals;
    const int64_t piece = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (piece >= pieces) return;
    const char *src = z + piece * 16;
    char *dst = y + piece * 16;
    auto frame_of = [&](int i) { return REVERSE ? T - 1 - i : i; };

    float ring[RING][NV];
#pragma unroll
    for (int r = 0; r < RING; ++r)
#pragma unroll
        for (int e = 0; e < NV; ++e) ring[r][e] = 0.0f;

    float next[NV];
    Vec<BF16>::load(next, src + (int64_t)frame_of(0) * frame_bytes);
    for (int tb = 0; tb < T; tb += RING) {
#pragma unroll
        for (int jj = 0; jj < RING; ++jj) {
            const int i = tb + jj;             // step; the frame it produces is t
            if (i < T) {
                const int t = frame_of(i);
#pragma unroll
                for (int e = 0; e < NV; ++e) ring[jj][e] = next[e];
                if (i + 1 < T) Vec<BF16>::load(next, src + (int64_t)frame_of(i + 1) * frame_bytes);   // before the store: y may be z
                const int terms = REVERSE ? min(w, T - t) : min(w, t + 1);
                const float uniform = 1.0f / (float)terms;
                float out[NV];
#pragma unroll
                for (int e = 0; e < NV; ++e) out[e] = 0.0f;
#pragma unroll
                for (int j = 0; j < RING; ++j) {
                    if (j < terms) {
                        const float c = m_band ? m_band[(int64_t)(REVERSE ? t + j : t) * w + j] : uniform;
#pragma unroll
                        for (int e = 0; e < NV; ++e) out[e] = fmaf(c, ring[(jj - j + RING) % RING][e], out[e]);
                    }
                }
                Vec<BF16>::store(dst + (int64_t)t * frame_bytes, out);
            }
        }
    }
}

// The paper's weights: ring of exactly W raw 16-byte pieces, running window sum in fp32.
// D frames are fetched ahead of the one being summed.  Every load is unconditional (beyond the last frame the
// last one is simply read again), so each is waited for by itself and a lane keeps D loads and its stores in
// flight; whole rounds of W steps run without a bounds test, the remainder of the series with one.
// REVERSE runs the adjoint, out_k = sum_{t=k}^{k+W-1} in_t / min(W, t): the time axis is walked from the end,
// a frame enters the running sum already divided by its own min(W, t) and leaves it the same way.
template <int W, bool BF16, bool REVERSE>
__global__ __launch_bounds__(kThreads) void mproduct_uniform_kernel(const char *z, char *y, int T, int64_t pieces,
                                                                    int64_t frame_bytes) {
    constexpr int NV = Vec<BF16>::kVals;
    constexpr int D = W % 4 == 0 ? 4 : (W % 2 == 0 ? 2 : 1);     // divides W, so a frame's queue slot is i % D = jj % D
    const int64_t piece = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (piece >= pieces) return;
    const char *src = z + piece * 16;
    char *dst = y + piece * 16;
    auto frame_of = [&](int i) { return REVERSE ? T - 1 - i : i; };

    uintx4 ring[W];
#pragma unroll
    for (int r = 0; r < W; ++r) ring[r] = uintx4{0u, 0u, 0u, 0u};   // the bit pattern of zeros in either type
    float sum[NV];
#pragma unroll
    for (int e = 0; e < NV; ++e) sum[e] = 0.0f;

    uintx4 ahead[D];
#pragma unroll
    for (int d = 0; d < D; ++d) ahead[d] = *reinterpret_cast<const uintx4 *>(src + (int64_t)frame_of(min(d, T - 1)) * frame_bytes);

    // one step i (0-based); `slot` holds the frame of step i - W, `queued` the frame of step i
    auto step = [&](int i, uintx4 &slot, uintx4 &queued) {
        const int t = frame_of(i);
        const uintx4 cur = queued;
        queued = *reinterpret_cast<const uintx4 *>(src + (int64_t)frame_of(min(i + D, T - 1)) * frame_bytes);   // before the store: y may be z
        float in[NV], old[NV], out[NV];
        Vec<BF16>::unpack(in, cur);
        Vec<BF16>::unpack(old, slot);
        slot = cur;
        const float scale = 1.0f / (float)min(W, t + 1);
#pragma unroll
        for (int e = 0; e < NV; ++e) {
            if (REVERSE) {
                sum[e] += in[e] * scale - old[e] * (1.0f / (float)W);    // the leaving frame is t + W: min(W, t + W + 1) = W
                out[e] = sum[e];
            } else {
                sum[e] += in[e] - old[e];
                out[e] = sum[e] * scale;
            }
        }
        Vec<BF16>::store(dst + (int64_t)t * frame_bytes, out);
    };
    int tb = 0;
    for (; tb + W <= T; tb += W) {
#pragma unroll
        for (int jj = 0; jj < W; ++jj) step(tb + jj, ring[jj], ahead[jj % D]);
    }
#pragma unroll
    for (int jj = 0; jj < W; ++jj)
        if (tb + jj < T) step(tb + jj, ring[jj], ahead[jj % D]);
}

template <int W, bool REVERSE>
int launch_uniform(const void *z, void *y, int64_t T, int64_t n, int32_t f, dgnn_dtype dt, hipStream_t s) {
    const int64_t frame_bytes = n * f * (dt == DGNN_F32 ? 4 : 2);
    const int64_t pieces = frame_bytes / 16;
    const unsigned blocks = (unsigned)((pieces + kThreads - 1) / kThreads);
    if (dt == DGNN_F32)
        hipLaunchKernelGGL((mproduct_uniform_kernel<W, false, REVERSE>), dim3(blocks), dim3(kThreads), 0, s,
                           static_cast<const char *>(z), static_cast<char *>(y), (int)T, pieces, frame_bytes);
    else
        hipLaunchKernelGGL((mproduct_uniform_kernel<W, true, REVERSE>), dim3(blocks), dim3(kThreads), 0, s,
                           static_cast<const char *>(z), static_cast<char *>(y), (int)T, pieces, frame_bytes);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

template <int W, bool REVERSE>
int dispatch_uniform(int w, const void *z, void *y, int64_t T, int64_t n, int32_t f, dgnn_dtype dt, hipStream_t s) {
    if (w == W) return launch_uniform<W, REVERSE>(z, y, T, n, f, dt, s);
    if constexpr (W > 1) return dispatch_uniform<W - 1, REVERSE>(w, z, y, T, n, f, dt, s);
    return DGNN_ERR_SHAPE;
}

template <int RING, bool REVERSE>
int launch(const void *z, void *y, int64_t T, int64_t n, int32_t f, int32_t w, const float *m_band, dgnn_dtype dt,
           hipStream_t s) {
    const int64_t frame_bytes = n * f * (dt == DGNN_F32 ? 4 : 2);
    const int64_t pieces = frame_bytes / 16;
    const unsigned blocks = (unsigned)((pieces + kThreads - 1) / kThreads);
    if (dt == DGNN_F32)
        hipLaunchKernelGGL((mproduct_kernel<RING, false, REVERSE>), dim3(blocks), dim3(kThreads), 0, s,
                           static_cast<const char *>(z), static_cast<char *>(y), (int)T, pieces, frame_bytes, (int)w, m_band);
    else
        hipLaunchKernelGGL((mproduct_kernel<RING, true, REVERSE>), dim3(blocks), dim3(kThreads), 0, s,
                           static_cast<const char *>(z), static_cast<char *>(y), (int)T, pieces, frame_bytes, (int)w, m_band);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

template <bool REVERSE>
int mproduct(const void *z, void *y, int64_t T, int64_t n, int32_t f, int32_t w, const float *m_band, dgnn_dtype dt,
             void *stream) {
    if (!z || !y) return DGNN_ERR_NULL;
    if (T <= 0 || n <= 0 || w <= 0 || !supported_width(f)) return DGNN_ERR_SHAPE;
    if (dt != DGNN_F32 && dt != DGNN_BF16) return DGNN_ERR_SHAPE;
    if (!fits_i32(n) || !fits_i32(T)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(z) || !aligned16(y)) return DGNN_ERR_ALIGN;
    const int64_t bytes = T * n * f * (dt == DGNN_F32 ? 4 : 2);
    if (y != z) {   // partial overlap is not allowed
        const char *a = static_cast<const char *>(z), *b = static_cast<const char *>(y);
        if (a < b + bytes && b < a + bytes) return DGNN_ERR_ALIAS;
    }
    // A window longer than the series acts like the series length; with explicit coefficients the
    // band layout keeps the caller's w as its row stride, so w itself must fit the ring.
    const int64_t eff = m_band ? (int64_t)w : (w < T ? (int64_t)w : T);
    if (eff > 32) return DGNN_ERR_SHAPE;
    const int32_t wk = m_band ? w : (int32_t)eff;
    hipStream_t s = (hipStream_t)stream;
    if (!m_band) return dispatch_uniform<32, REVERSE>((int)eff, z, y, T, n, f, dt, s);
    if (eff <= 4) return launch<4, REVERSE>(z, y, T, n, f, wk, m_band, dt, s);
    if (eff <= 8) return launch<8, REVERSE>(z, y, T, n, f, wk, m_band, dt, s);
    if (eff <= 16) return launch<16, REVERSE>(z, y, T, n, f, wk, m_band, dt, s);
    return launch<32, REVERSE>(z, y, T, n, f, wk, m_band, dt, s);
}

}  // namespace

extern "C" int dgnn_mproduct(const void *z, void *y, int64_t T, int64_t n, int32_t f, int32_t w,
                             const float *m_band, dgnn_dtype dt, void *stream) {
    return mproduct<false>(z, y, T, n, f, w, m_band, dt, stream);
}

extern "C" int dgnn_mproduct_backward(const void *g_y, void *g_z, int64_t T, int64_t n, int32_t f, int32_t w,
                                      const float *m_band, dgnn_dtype dt, void *stream) {
    return mproduct<true>(g_y, g_z, T, n, f, w, m_band, dt, stream);
}
