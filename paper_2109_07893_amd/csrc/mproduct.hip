// M-transform of TM-GCN (Section "TM-GCN"): Y = Z x_1 M with the banded lower-triangular M,
//     Y_t = sum_{j=0}^{min(w,t)-1} m(t,j) Z_{t-j},   m(t,j) = 1/min(w,t) unless given.
//
// Each lane owns one 16-byte piece of the N x F frame and walks the time axis once, keeping the
// last w frames of its piece in a register ring, so every frame is read once and written once
// (2 s N F bytes per timestep) whatever the window, and the transform can run in place.
// The time loop is unrolled by the ring size so that ring slots are compile-time registers.
// With the paper's weights (every term 1/min(w,t)) the window sum is kept as a running sum,
// S_t = S_{t-1} + Z_t - Z_{t-w}, with a ring of exactly w slots (the slot about to be overwritten
// holds Z_{t-w}) and up to four frames fetched ahead; every w steps the sum is replaced by one formed
// from that round's frames alone, so that what a frame leaves behind in it (rounding residue, or
// not-a-number once an infinity has left the window) is gone less than two windows later.  Explicit
// coefficients take the general kernels, w multiply-adds per element.
//
// A series longer than one block of timesteps is mixed block by block (Section "Gradient Checkpoint": what a
// block needs from the one before it is handed over).  Going forward the hand-over is the last w - 1 frames
// before the block, going back the first w - 1 gradient frames after it; either way they are put into the ring
// before the walk begins, as if the walk had just passed them, and t0 (the number of timesteps before the
// block) enters the weights 1/min(w, t).
#include "common.hpp"

namespace {

using namespace dgnn;

// Frames handed over from the neighbouring block: `count` frames of the block's shape, the nearest LAST going
// forward (oldest first) and the nearest FIRST going back; t0 = timesteps before the block.
struct Halo {
    const char *frames;
    int count;
    int t0;
};

typedef float floatx4 __attribute__((ext_vector_type(4)));

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
        __builtin_nontemporal_store(floatx4{v[0], v[1], v[2], v[3]}, reinterpret_cast<floatx4 *>(p));   // every frame is read once and written once: a stream
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
        __builtin_nontemporal_store(t, reinterpret_cast<uintx4 *>(p));
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
                                                            int64_t frame_bytes, int w, const float *__restrict__ m_band,
                                                            Halo halo) {
    constexpr int NV = Vec<BF16>::kVals;
    const int64_t piece = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (piece >= pieces) return;
    const char *src = z + piece * 16;
    char *dst = y + piece * 16;
    auto frame_of = [&](int i) { return REVERSE ? T - 1 - i : i; };

    // slot r of the ring is where step (r - RING) would have left its frame: the handed-over frames go there
    float ring[RING][NV];
#pragma unroll
    for (int r = 0; r < RING; ++r) {
#pragma unroll
        for (int e = 0; e < NV; ++e) ring[r][e] = 0.0f;
        const int h = REVERSE ? RING - 1 - r : halo.count - (RING - r);
        if (h >= 0 && h < halo.count) Vec<BF16>::load(ring[r], halo.frames + (int64_t)h * frame_bytes + piece * 16);
    }

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
                const int terms = REVERSE ? min(w, T - t + halo.count) : min(w, t + 1 + halo.count);
                const float uniform = 1.0f / (float)min(w, halo.t0 + t + 1);
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

// The same with explicit coefficients for rings too long for the kernel above (its body, unrolled over ring slots
// times window terms, grows with the square of the ring, and the compiler then keeps the ring in scratch memory):
// the ring holds raw 16-byte pieces, slot j always the frame of j steps ago, and moves down one slot per step, so
// every slot is a fixed register and the body grows with the ring only.
template <int RING, bool BF16, bool REVERSE>
__global__ __launch_bounds__(kThreads) void mproduct_shift_kernel(const char *z, char *y, int T, int64_t pieces,
                                                                  int64_t frame_bytes, int w, const float *__restrict__ m_band,
                                                                  Halo halo) {
    constexpr int NV = Vec<BF16>::kVals;
    const int64_t piece = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (piece >= pieces) return;
    const char *src = z + piece * 16;
    char *dst = y + piece * 16;
    auto frame_of = [&](int i) { return REVERSE ? T - 1 - i : i; };

    // before the first step, slot j - 1 holds the frame of step -j: a handed-over frame, or nothing
    uintx4 ring[RING];
#pragma unroll
    for (int j = 1; j <= RING; ++j) {
        ring[j - 1] = uintx4{0u, 0u, 0u, 0u};
        const int h = REVERSE ? j - 1 : halo.count - j;
        if (h >= 0 && h < halo.count) ring[j - 1] = *reinterpret_cast<const uintx4 *>(halo.frames + (int64_t)h * frame_bytes + piece * 16);
    }
    uintx4 next = __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(src + (int64_t)frame_of(0) * frame_bytes));
#pragma unroll 1
    for (int i = 0; i < T; ++i) {
        const int t = frame_of(i);
#pragma unroll
        for (int j = RING - 1; j > 0; --j) ring[j] = ring[j - 1];
        ring[0] = next;
        next = __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(src + (int64_t)frame_of(min(i + 1, T - 1)) * frame_bytes));   // before the store: y may be z
        const int terms = REVERSE ? min(w, T - t + halo.count) : min(w, t + 1 + halo.count);
        float out[NV];
#pragma unroll
        for (int e = 0; e < NV; ++e) out[e] = 0.0f;
#pragma unroll
        for (int j = 0; j < RING; ++j) {
            if (j < terms) {
                const float c = m_band[(int64_t)(REVERSE ? t + j : t) * w + j];
                float v[NV];
                Vec<BF16>::unpack(v, ring[j]);
#pragma unroll
                for (int e = 0; e < NV; ++e) out[e] = fmaf(c, v[e], out[e]);
            }
        }
        Vec<BF16>::store(dst + (int64_t)t * frame_bytes, out);
    }
}

// The paper's weights: ring of exactly W raw 16-byte pieces, running window sum in fp32.
// D frames are fetched ahead of the one being summed.  Every load is unconditional (beyond the last frame the
// last one is simply read again), so each is waited for by itself and a lane keeps D loads and its stores in
// flight; whole rounds of W steps run without a bounds test, the remainder of the series with one.
// REVERSE runs the adjoint, out_k = sum_{t=k}^{k+W-1} in_t / min(W, t): the time axis is walked from the end,
// a frame enters the running sum already divided by its own min(W, t) and leaves it the same way.
// Wavefronts per SIMD the compiler must leave room for.  Left to itself it spends 232 registers on the unrolled
// round of a 16-frame window in bf16 (two wavefronts per SIMD: too few loads in flight for an in-place stream);
// held to 168 (three per SIMD) it spills three values outside the loop and the in-place transform runs an eighth
// faster.  Only where that is all it costs: the adjoint and windows beyond 23 frames would spill inside the loop,
// fp32 and the shorter windows fit three wavefronts anyway.
constexpr int uniform_waves_per_simd(int w, bool bf16, bool reverse) { return (bf16 && !reverse && w >= 12 && w <= 23) ? 3 : 1; }

template <int W, bool BF16, bool REVERSE>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(uniform_waves_per_simd(W, BF16, REVERSE))))
void mproduct_uniform_kernel(const char *z, char *y, int T, int64_t pieces,
                                                                    int64_t frame_bytes, Halo halo) {
    constexpr int NV = Vec<BF16>::kVals;
    constexpr int D = W % 4 == 0 ? 4 : (W % 2 == 0 ? 2 : 1);     // divides W, so a frame's queue slot is i % D = jj % D
    const int64_t piece = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (piece >= pieces) return;
    const char *src = z + piece * 16;
    char *dst = y + piece * 16;
    auto frame_of = [&](int i) { return REVERSE ? T - 1 - i : i; };

    uintx4 ring[W];
    float sum[NV], fresh[NV];          // the running window sum, and the sum of the frames of the current round
#pragma unroll
    for (int e = 0; e < NV; ++e) sum[e] = fresh[e] = 0.0f;
    // slot r of the ring is where step (r - W) would have left its frame: the handed-over frames go there and
    // into the running sum
#pragma unroll
    for (int r = 0; r < W; ++r) {
        ring[r] = uintx4{0u, 0u, 0u, 0u};   // the bit pattern of zeros in either type
        const int h = REVERSE ? W - 1 - r : halo.count - (W - r);
        if (h >= 0 && h < halo.count) {
            ring[r] = *reinterpret_cast<const uintx4 *>(halo.frames + (int64_t)h * frame_bytes + piece * 16);
            float v[NV];
            Vec<BF16>::unpack(v, ring[r]);
            const float sc = REVERSE ? 1.0f / (float)min(W, halo.t0 + T + h + 1) : 1.0f;
#pragma unroll
            for (int e = 0; e < NV; ++e) sum[e] += v[e] * sc;
        }
    }

    uintx4 ahead[D];
#pragma unroll
    for (int d = 0; d < D; ++d) ahead[d] = __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(src + (int64_t)frame_of(min(d, T - 1)) * frame_bytes));

    // one step i (0-based); `slot` holds the frame of step i - W, `queued` the frame of step i
    auto step = [&](int i, uintx4 &slot, uintx4 &queued) {
        const int t = frame_of(i);
        const uintx4 cur = queued;
        queued = __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(src + (int64_t)frame_of(min(i + D, T - 1)) * frame_bytes));   // before the store: y may be z
        float in[NV], old[NV], out[NV];
        Vec<BF16>::unpack(in, cur);
        Vec<BF16>::unpack(old, slot);
        slot = cur;
        const float scale = 1.0f / (float)min(W, halo.t0 + t + 1);
#pragma unroll
        for (int e = 0; e < NV; ++e) {
            if (REVERSE) {
                sum[e] += in[e] * scale - old[e] * (1.0f / (float)W);    // the leaving frame is t + W: min(W, t + W + 1) = W
                fresh[e] += in[e] * scale;
                out[e] = sum[e];
            } else {
                sum[e] += in[e] - old[e];
                fresh[e] += in[e];
                out[e] = sum[e] * scale;
            }
        }
        Vec<BF16>::store(dst + (int64_t)t * frame_bytes, out);
    };
    int tb = 0;
    for (; tb + W <= T; tb += W) {
#pragma unroll
        for (int e = 0; e < NV; ++e) fresh[e] = 0.0f;
#pragma unroll
        for (int jj = 0; jj < W; ++jj) step(tb + jj, ring[jj], ahead[jj % D]);
        // A whole round has gone by: the W frames it brought in are exactly the window now, and `fresh` is their sum
        // formed on its own.  It replaces the running sum, so that rounding residue of large values, and anything
        // that is not a number, stop travelling along here instead of staying in the sum for the rest of the series.
#pragma unroll
        for (int e = 0; e < NV; ++e) sum[e] = fresh[e];
    }
#pragma unroll
    for (int jj = 0; jj < W; ++jj)
        if (tb + jj < T) step(tb + jj, ring[jj], ahead[jj % D]);
}

template <int W, bool REVERSE>
int launch_uniform(const void *z, void *y, int64_t T, int64_t n, int32_t f, dgnn_dtype dt, Halo halo, hipStream_t s) {
    const int64_t frame_bytes = n * f * (dt == DGNN_F32 ? 4 : 2);
    const int64_t pieces = frame_bytes / 16;
    const unsigned blocks = (unsigned)((pieces + kThreads - 1) / kThreads);
    if (dt == DGNN_F32)
        hipLaunchKernelGGL((mproduct_uniform_kernel<W, false, REVERSE>), dim3(blocks), dim3(kThreads), 0, s,
                           static_cast<const char *>(z), static_cast<char *>(y), (int)T, pieces, frame_bytes, halo);
    else
        hipLaunchKernelGGL((mproduct_uniform_kernel<W, true, REVERSE>), dim3(blocks), dim3(kThreads), 0, s,
                           static_cast<const char *>(z), static_cast<char *>(y), (int)T, pieces, frame_bytes, halo);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

template <int W, bool REVERSE>
int dispatch_uniform(int w, const void *z, void *y, int64_t T, int64_t n, int32_t f, dgnn_dtype dt, Halo halo,
                     hipStream_t s) {
    if (w == W) return launch_uniform<W, REVERSE>(z, y, T, n, f, dt, halo, s);
    if constexpr (W > 1) return dispatch_uniform<W - 1, REVERSE>(w, z, y, T, n, f, dt, halo, s);
    return DGNN_ERR_SHAPE;
}

template <int RING, bool REVERSE>
int launch(const void *z, void *y, int64_t T, int64_t n, int32_t f, int32_t w, const float *m_band, dgnn_dtype dt,
           Halo halo, hipStream_t s) {
    const int64_t frame_bytes = n * f * (dt == DGNN_F32 ? 4 : 2);
    const int64_t pieces = frame_bytes / 16;
    const unsigned blocks = (unsigned)((pieces + kThreads - 1) / kThreads);
    if (dt == DGNN_F32)
        hipLaunchKernelGGL((mproduct_kernel<RING, false, REVERSE>), dim3(blocks), dim3(kThreads), 0, s,
                           static_cast<const char *>(z), static_cast<char *>(y), (int)T, pieces, frame_bytes, (int)w, m_band, halo);
    else
        hipLaunchKernelGGL((mproduct_kernel<RING, true, REVERSE>), dim3(blocks), dim3(kThreads), 0, s,
                           static_cast<const char *>(z), static_cast<char *>(y), (int)T, pieces, frame_bytes, (int)w, m_band, halo);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

template <int RING, bool REVERSE>
int launch_shift(const void *z, void *y, int64_t T, int64_t n, int32_t f, int32_t w, const float *m_band, dgnn_dtype dt,
                 Halo halo, hipStream_t s) {
    const int64_t frame_bytes = n * f * (dt == DGNN_F32 ? 4 : 2);
    const int64_t pieces = frame_bytes / 16;
    const unsigned blocks = (unsigned)((pieces + kThreads - 1) / kThreads);
    if (dt == DGNN_F32)
        hipLaunchKernelGGL((mproduct_shift_kernel<RING, false, REVERSE>), dim3(blocks), dim3(kThreads), 0, s,
                           static_cast<const char *>(z), static_cast<char *>(y), (int)T, pieces, frame_bytes, (int)w, m_band, halo);
    else
        hipLaunchKernelGGL((mproduct_shift_kernel<RING, true, REVERSE>), dim3(blocks), dim3(kThreads), 0, s,
                           static_cast<const char *>(z), static_cast<char *>(y), (int)T, pieces, frame_bytes, (int)w, m_band, halo);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

template <bool REVERSE>
int mproduct(const void *z, void *y, int64_t T, int64_t n, int32_t f, int32_t w, const float *m_band, int64_t t0,
             const void *halo_frames, int64_t n_halo, dgnn_dtype dt, void *stream) {
    if (!z || !y) return DGNN_ERR_NULL;
    if (T <= 0 || n <= 0 || w <= 0 || t0 < 0 || n_halo < 0 || !supported_width(f)) return DGNN_ERR_SHAPE;
    if (dt != DGNN_F32 && dt != DGNN_BF16) return DGNN_ERR_SHAPE;
    if (!fits_index(n) || !fits_i32(T) || !fits_i32(t0 + T + n_halo)) return DGNN_ERR_OVERFLOW;
    if (n_halo > 0 && !halo_frames) return DGNN_ERR_NULL;
    if (n_halo > w - 1) return DGNN_ERR_SHAPE;
    if (!REVERSE && n_halo != (t0 < w - 1 ? t0 : w - 1)) return DGNN_ERR_SHAPE;   // exactly the frames the window reaches
    if (!aligned16(z) || !aligned16(y) || !aligned16(halo_frames)) return DGNN_ERR_ALIGN;
    const int64_t frame = n * f * (dt == DGNN_F32 ? 4 : 2);
    const int64_t bytes = T * frame;
    const char *a = static_cast<const char *>(z), *b = static_cast<const char *>(y);
    if (y != z && a < b + bytes && b < a + bytes) return DGNN_ERR_ALIAS;             // partial overlap is not allowed
    if (n_halo > 0) {
        const char *h = static_cast<const char *>(halo_frames);
        if (h < b + bytes && b < h + n_halo * frame) return DGNN_ERR_ALIAS;           // the output would overwrite the hand-over
    }
    // The ring holds min(w, length of the series so far) frames; with explicit coefficients the band layout
    // keeps the caller's w as its row stride, so w itself must fit the ring.
    const int64_t seen = t0 + T + (REVERSE ? n_halo : 0);
    const int64_t eff = m_band ? (int64_t)w : (w < seen ? (int64_t)w : seen);
    if (eff > 32) return DGNN_ERR_SHAPE;
    const int32_t wk = m_band ? w : (int32_t)eff;
    const Halo halo{static_cast<const char *>(halo_frames), (int)n_halo, (int)t0};
    hipStream_t s = (hipStream_t)stream;
    if (!m_band) return dispatch_uniform<32, REVERSE>((int)eff, z, y, T, n, f, dt, halo, s);
    if (eff <= 4) return launch<4, REVERSE>(z, y, T, n, f, wk, m_band, dt, halo, s);
    if (eff <= 8) return launch<8, REVERSE>(z, y, T, n, f, wk, m_band, dt, halo, s);
    if (eff <= 16) return launch<16, REVERSE>(z, y, T, n, f, wk, m_band, dt, halo, s);
    if (eff <= 24) return launch_shift<24, REVERSE>(z, y, T, n, f, wk, m_band, dt, halo, s);
    return launch_shift<32, REVERSE>(z, y, T, n, f, wk, m_band, dt, halo, s);
}

}  // namespace

extern "C" int dgnn_mproduct(const void *z, void *y, int64_t T, int64_t n, int32_t f, int32_t w,
                             const float *m_band, dgnn_dtype dt, void *stream) {
    return mproduct<false>(z, y, T, n, f, w, m_band, 0, nullptr, 0, dt, stream);
}

extern "C" int dgnn_mproduct_backward(const void *g_y, void *g_z, int64_t T, int64_t n, int32_t f, int32_t w,
                                      const float *m_band, dgnn_dtype dt, void *stream) {
    return mproduct<true>(g_y, g_z, T, n, f, w, m_band, 0, nullptr, 0, dt, stream);
}

extern "C" int dgnn_mproduct_block(const void *z, void *y, int64_t T, int64_t n, int32_t f, int32_t w,
                                   const float *m_band, int64_t t0, const void *z_before, int64_t n_before,
                                   dgnn_dtype dt, void *stream) {
    return mproduct<false>(z, y, T, n, f, w, m_band, t0, z_before, n_before, dt, stream);
}

extern "C" int dgnn_mproduct_backward_block(const void *g_y, void *g_z, int64_t T, int64_t n, int32_t f, int32_t w,
                                            const float *m_band, int64_t t0, const void *g_after, int64_t n_after,
                                            dgnn_dtype dt, void *stream) {
    return mproduct<true>(g_y, g_z, T, n, f, w, m_band, t0, g_after, n_after, dt, stream);
}
