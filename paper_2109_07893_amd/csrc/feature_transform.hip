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
// row: step s of the fp32 kernel multiplies k = h F/2 + s, step s of the bf16 kernel the eight
// values k = h F/2 + 8 s .. + 7.  The accumulator of a 32x32 tile holds, in register v of lane
// l, the element (row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32).
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
    for (int64_t tile = (int64_t)blockIdx.x * kWavesPerBlock + wave; tile < n_tiles;
         tile += (int64_t)gridDim.x * kWavesPerBlock) {
        const int64_t row = tile * 32 + i;
        floatx4 a[KH / 4];
        if (row < n) {
            const floatx4 *src = reinterpret_cast<const floatx4 *>(x + row * FIN + hh * KH);
#pragma unroll
            for (int q = 0; q < KH / 4; ++q) a[q] = src[q];
        } else {
#pragma unroll
            for (int q = 0; q < KH / 4; ++q) a[q] = floatx4{0.f, 0.f, 0.f, 0.f};
        }
        floatx16 acc[NT];
#pragma unroll
        for (int jt = 0; jt < NT; ++jt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[jt][v] = 0.0f;
#pragma unroll
        for (int s = 0; s < KH; ++s) {
            const float av = a[s / 4][s % 4];
#pragma unroll
            for (int jt = 0; jt < NT; ++jt) {
                const float bv = s_w[(hh * KH + s) * LD + jt * 32 + i];
                acc[jt] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[jt], 0, 0, 0);
            }
        }
        float scale[16];   // row_scale of the 16 rows this lane stores: one coalesced load, then lane exchange
        {
            const float mine = (row_scale && row < n) ? row_scale[row] : 1.0f;   // lane (i, hh) holds row i
#pragma unroll
            for (int v = 0; v < 16; ++v) scale[v] = __shfl(mine, 8 * (v / 4) + 4 * hh + (v % 4), kWave);
        }
#pragma unroll
        for (int jt = 0; jt < NT; ++jt) {
            const int col = jt * 32 + i;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t r = tile * 32 + 8 * (v / 4) + 4 * hh + (v % 4);
                if (r < n && col < FOUT) h[r * FOUT + col] = acc[jt][v] * scale[v];
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
    for (int64_t tile = (int64_t)blockIdx.x * kWavesPerBlock + wave; tile < n_tiles;
         tile += (int64_t)gridDim.x * kWavesPerBlock) {
        const int64_t row = tile * 32 + i;
        bf16x8 a[KS];
        if (row < n) {
            const bf16x8 *src = reinterpret_cast<const bf16x8 *>(x + row * FIN + hh * KH);
#pragma unroll
            for (int s = 0; s < KS; ++s) a[s] = src[s];
        } else {
#pragma unroll
            for (int s = 0; s < KS; ++s)
#pragma unroll
                for (int e = 0; e < 8; ++e) a[s][e] = (__bf16)0.0f;
        }
        floatx16 acc[NT];
#pragma unroll
        for (int jt = 0; jt < NT; ++jt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[jt][v] = 0.0f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
#pragma unroll
            for (int jt = 0; jt < NT; ++jt) {
                const bf16x8 bv = *reinterpret_cast<const bf16x8 *>(&s_wt[(jt * 32 + i) * LDW + hh * KH + s * 8]);
                acc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s], bv, acc[jt], 0, 0, 0);
            }
        }
        float scale[16];   // row_scale of the 16 rows this lane stores: one coalesced load, then lane exchange
        {
            const float mine = (row_scale && row < n) ? row_scale[row] : 1.0f;   // lane (i, hh) holds row i
#pragma unroll
            for (int v = 0; v < 16; ++v) scale[v] = __shfl(mine, 8 * (v / 4) + 4 * hh + (v % 4), kWave);
        }
#pragma unroll
        for (int jt = 0; jt < NT; ++jt) {
            const int col = jt * 32 + i;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t r = tile * 32 + 8 * (v / 4) + 4 * hh + (v % 4);
                if (r < n && col < FOUT) h[r * FOUT + col] = (uint16_t)f32_to_bf16(acc[jt][v] * scale[v]);
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
