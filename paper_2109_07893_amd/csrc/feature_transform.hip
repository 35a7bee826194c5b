// Dense factor of the GCN operation, Eqn (2): H = X W on the gfx950 matrix cores.
//
// The product is HBM-bound (2 F F' flops per row against s (F + F') bytes), so the kernel is
// shaped as a stream: W is parked in LDS once per workgroup, each wavefront takes 32 rows of X
// per iteration, every lane reads one contiguous half row straight from global memory into
// the A operand registers, and the 32x32 accumulator tiles are stored row-wise.
//
// Operand mapping.  In a 32x32xK MFMA, lane l supplies row (l % 32) of A and column (l % 32)
// of B for the k-slice selected by h = l / 32.  The order in which k is consumed is free as
// long as A and B agree, so lane (i, h) owns the contiguous k range [h F/2, (h+1) F/2) of its
// row of X: step s of the fp32 kernel multiplies k = h F/2 + s, step s of the bf16 kernel the
// eight values k = h F/2 + 8 s .. + 7.  The accumulator of a 32x32 tile holds, in register v of
// lane l, the element (row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32).  The fp32 kernel
// stores that layout as it is: per register the two lane halves write two whole 128-byte lines.
// The bf16 kernel computes the TRANSPOSED tile, (X W)^T = W^T X^T, with W^T as the A operand and
// the rows of X as the B operand: lane (i, h) then holds row i of the result and, in every four
// consecutive accumulator registers, four consecutive columns of it, which turns sixty-four
// 2-byte stores per lane into sixteen 8-byte ones and makes row_scale one value per lane.
#include "common.hpp"

namespace {

using namespace dgnn;

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / kWave;

template <int FIN, int FOUT>
__global__ __launch_bounds__(kThreads) void xw_f32_kernel(const float *__restrict__ x, const float *__restrict__ w,
                                                          const float *__restrict__ row_scale, float *__restrict__ h,
                                                          int64_t n, int64_t n_tiles) {
    constexpr int NT = (FOUT + 31) / 32;   // 32-wide column tiles (FOUT = 16 is zero-padded)
    constexpr int LD = NT * 32;
    constexpr int KH = FIN / 2;            // k values owned by one lane
    __shared__ float s_w[FIN * LD];

    const int tid = threadIdx.x;
    for (int idx = tid; idx < FIN * LD; idx += kThreads) {
        int k = idx / LD, j = idx % LD;
        s_w[idx] = j < FOUT ? w[k * FOUT + j] : 0.0f;
    }
    __syncthreads();

    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int i = lane & 31, hh = lane >> 5;
    const int64_t stride = (int64_t)gridDim.x * kWavesPerBlock;
    int64_t tile = (int64_t)blockIdx.x * kWavesPerBlock + wave;

    floatx4 a_next[KH / 4];
    float sc_next = 1.0f;
    auto fetch = [&](int64_t t) {
        const int64_t row = t * 32 + i;
        if (t < n_tiles && row < n) {
            const floatx4 *src = reinterpret_cast<const floatx4 *>(x + row * FIN + hh * KH);
#pragma unroll
            for (int q = 0; q < KH / 4; ++q) a_next[q] = src[q];
            sc_next = row_scale ? row_scale[row] : 1.0f;
        } else {
#pragma unroll
            for (int q = 0; q < KH / 4; ++q) a_next[q] = floatx4{0.f, 0.f, 0.f, 0.f};
        }
    };
    fetch(tile);
    for (; tile < n_tiles; tile += stride) {
        floatx4 a[KH / 4];
#pragma unroll
        for (int q = 0; q < KH / 4; ++q) a[q] = a_next[q];
        const float scale = sc_next;
        fetch(tile + stride);              // the next tile's rows travel while this one is multiplied
        floatx16 acc[NT];
#pragma unroll
        for (int jt = 0; jt < NT; ++jt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[jt][v] = 0.0f;
#pragma unroll
        for (int s = 0; s < KH; ++s) {
            const float xv = a[s / 4][s % 4];
#pragma unroll
            for (int jt = 0; jt < NT; ++jt) {
                const float wv = s_w[(hh * KH + s) * LD + jt * 32 + i];
                acc[jt] = __builtin_amdgcn_mfma_f32_32x32x2f32(xv, wv, acc[jt], 0, 0, 0);
            }
        }
        // register v of lane (i, hh) holds row 8 (v / 4) + 4 hh + v % 4, column i of the tile: per register the
        // two lane halves write two whole 128-byte rows
        float sc[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) sc[v] = __shfl(scale, 8 * (v / 4) + 4 * hh + (v % 4), kWave);
#pragma unroll
        for (int jt = 0; jt < NT; ++jt) {
            const int col = jt * 32 + i;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t r = tile * 32 + 8 * (v / 4) + 4 * hh + (v % 4);
                if (r < n && col < FOUT) h[r * FOUT + col] = acc[jt][v] * sc[v];
            }
        }
    }
}

template <int FIN, int FOUT>
__global__ __launch_bounds__(kThreads) void xw_bf16_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ w,
                                                           const float *__restrict__ row_scale, uint16_t *__restrict__ h,
                                                           int64_t n, int64_t n_tiles) {
    constexpr int NT = (FOUT + 31) / 32;
    constexpr int KH = FIN / 2;            // bf16 values owned by one lane
    constexpr int KS = KH / 8;             // MFMA steps of depth 16 (8 per lane half)
    constexpr int LDW = FIN + 8;           // padded row of W^T in LDS, keeps 16-byte reads conflict-free
    __shared__ __attribute__((aligned(16))) uint16_t s_wt[NT * 32 * LDW];   // W transposed: [column][k]

    const int tid = threadIdx.x;
    for (int idx = tid; idx < FIN * NT * 32; idx += kThreads) {
        int k = idx / (NT * 32), j = idx % (NT * 32);
        s_wt[j * LDW + k] = j < FOUT ? w[k * FOUT + j] : (uint16_t)0;
    }
    __syncthreads();

    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int i = lane & 31, hh = lane >> 5;
    const int64_t stride = (int64_t)gridDim.x * kWavesPerBlock;
    int64_t tile = (int64_t)blockIdx.x * kWavesPerBlock + wave;

    bf16x8 a_next[KS];
    float sc_next = 1.0f;
    auto fetch = [&](int64_t t) {
        const int64_t row = t * 32 + i;
        if (t < n_tiles && row < n) {
            const bf16x8 *src = reinterpret_cast<const bf16x8 *>(x + row * FIN + hh * KH);
#pragma unroll
            for (int s = 0; s < KS; ++s) a_next[s] = src[s];
            sc_next = row_scale ? row_scale[row] : 1.0f;
        } else {
#pragma unroll
            for (int s = 0; s < KS; ++s)
#pragma unroll
                for (int e = 0; e < 8; ++e) a_next[s][e] = (__bf16)0.0f;
        }
    };
    fetch(tile);
    for (; tile < n_tiles; tile += stride) {
        bf16x8 a[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) a[s] = a_next[s];
        const float scale = sc_next;
        fetch(tile + stride);
        floatx16 acc[NT];
#pragma unroll
        for (int jt = 0; jt < NT; ++jt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[jt][v] = 0.0f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
#pragma unroll
            for (int jt = 0; jt < NT; ++jt) {
                const bf16x8 wv = *reinterpret_cast<const bf16x8 *>(&s_wt[(jt * 32 + i) * LDW + hh * KH + s * 8]);
                acc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, a[s], acc[jt], 0, 0, 0);   // (X W)^T tile
            }
        }
        const int64_t row = tile * 32 + i;
        if (row < n) {
#pragma unroll
            for (int jt = 0; jt < NT; ++jt)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int col = jt * 32 + 8 * g + 4 * hh;
                    if (col < FOUT) {
                        const uint32_t lo = f32_to_bf16(acc[jt][4 * g] * scale) | (f32_to_bf16(acc[jt][4 * g + 1] * scale) << 16);
                        const uint32_t hi = f32_to_bf16(acc[jt][4 * g + 2] * scale) | (f32_to_bf16(acc[jt][4 * g + 3] * scale) << 16);
                        *reinterpret_cast<uint2 *>(h + row * FOUT + col) = make_uint2(lo, hi);
                    }
                }
        }
    }
}

template <int FIN, int FOUT>
int launch(const void *x, const void *w, const float *row_scale, void *h, int64_t n, dgnn_dtype dt, hipStream_t s) {
    const int64_t n_tiles = (n + 31) / 32;
    int64_t blocks = (n_tiles + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > 4096) blocks = 4096;
    if (dt == DGNN_F32) {
        hipLaunchKernelGGL((xw_f32_kernel<FIN, FOUT>), dim3((unsigned)blocks), dim3(kThreads), 0, s,
                           static_cast<const float *>(x), static_cast<const float *>(w), row_scale, static_cast<float *>(h), n, n_tiles);
    } else {
        hipLaunchKernelGGL((xw_bf16_kernel<FIN, FOUT>), dim3((unsigned)blocks), dim3(kThreads), 0, s,
                           static_cast<const uint16_t *>(x), static_cast<const uint16_t *>(w), row_scale,
                           static_cast<uint16_t *>(h), n, n_tiles);
    }
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

template <int FIN>
int launch_out(int32_t f_out, const void *x, const void *w, const float *row_scale, void *h, int64_t n, dgnn_dtype dt,
               hipStream_t s) {
    switch (f_out) {
        case 16: return launch<FIN, 16>(x, w, row_scale, h, n, dt, s);
        case 32: return launch<FIN, 32>(x, w, row_scale, h, n, dt, s);
        case 64: return launch<FIN, 64>(x, w, row_scale, h, n, dt, s);
        case 128: return launch<FIN, 128>(x, w, row_scale, h, n, dt, s);
        default: return DGNN_ERR_SHAPE;
    }
}

}  // namespace

extern "C" int dgnn_feature_transform(const void *x, int64_t n, int32_t f_in, const void *w, int32_t f_out,
                                      const float *row_scale, void *h, dgnn_dtype dt, void *stream) {
    if (!x || !w || !h) return DGNN_ERR_NULL;
    if (n <= 0 || !supported_width(f_in) || !supported_width(f_out)) return DGNN_ERR_SHAPE;
    if (dt != DGNN_F32 && dt != DGNN_BF16) return DGNN_ERR_SHAPE;
    if (!fits_i32(n)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(x) || !aligned16(h)) return DGNN_ERR_ALIGN;
    if (x == h) return DGNN_ERR_ALIAS;
    hipStream_t s = (hipStream_t)stream;
    switch (f_in) {
        case 16: return launch_out<16>(f_out, x, w, row_scale, h, n, dt, s);
        case 32: return launch_out<32>(f_out, x, w, row_scale, h, n, dt, s);
        case 64: return launch_out<64>(f_out, x, w, row_scale, h, n, dt, s);
        case 128: return launch_out<128>(f_out, x, w, row_scale, h, n, dt, s);
        default: return DGNN_ERR_SHAPE;
    }
}
