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
//
// Where W and one 32-row tile per wavefront fit in LDS together (fp32 up to width 64, bf16 from width 32 on)
// the "staged" kernels are used instead: a tile is read from global memory as consecutive 16-byte pieces,
// laid down in LDS with padded rows, picked up in operand layout, and the result goes back the same way,
// so that every global access of a wavefront is a run of whole lines.  The direct kernels serve the rest.
// A tile buffer belongs to one wavefront, so its phases are ordered by wavefront-level LDS synchronisation, not by
// workgroup barriers: the wavefronts of a workgroup drift apart and one multiplies while another moves data.
// Every kernel walks its tiles with a stride of the whole grid; the launch decides how many tiles a wavefront gets.
#include <algorithm>

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
                                                          int64_t n, int64_t n_tiles, int wt) {
    constexpr int NT = (FOUT + 31) / 32;   // 32-wide column tiles (FOUT = 16 is zero-padded)
    constexpr int LD = NT * 32;
    constexpr int KH = FIN / 2;            // k values owned by one lane
    __shared__ float s_w[FIN * LD];

    const int tid = threadIdx.x;
    for (int idx = tid; idx < FIN * LD; idx += kThreads) {
        int k = idx / LD, j = idx % LD;
        s_w[idx] = j < FOUT ? w[wt ? j * FIN + k : k * FOUT + j] : 0.0f;
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

// The same product with both tiles staged through LDS, for widths whose tiles fit: the 32 rows of X arrive as
// one contiguous block (every load instruction of the wavefront covers whole 128-byte lines), are laid down
// in LDS with padded rows and picked up again in operand order; the result tile takes the same way back, so
// the stores are whole lines too.  The product is computed transposed, (X W)^T = W^T X^T, which leaves lane
// (i, h) with row i of the result and four consecutive columns in every four accumulator registers.
// CONCAT: the output row is relu([x | x W]), FIN + FOUT wide (the skip connection of the CD-GCN layer, Section
// "CD-GCN"): the result tile is laid down behind the input tile, which is still in LDS, and both leave together.
template <int FIN, int FOUT, bool CONCAT>
__global__ __launch_bounds__(kThreads) void xw_f32_staged_kernel(const float *__restrict__ x, const float *__restrict__ w,
                                                                 const float *__restrict__ row_scale, float *__restrict__ h,
                                                                 int64_t n, int64_t n_tiles, int wt) {
    constexpr int NT = FOUT / 32;
    constexpr int KH = FIN / 2;
    constexpr int FMAX = FIN > FOUT ? FIN : FOUT;
    constexpr int ROFF = CONCAT ? FIN : 0;           // where the result begins in a staged row
    constexpr int OUTW = CONCAT ? FIN + FOUT : FOUT; // width of an output row
    constexpr int LDT = (CONCAT ? FIN + FOUT : FMAX) + 4;   // padded tile row (floats): 16 bytes of padding
    constexpr int IN_PIECES = 32 * FIN / 4 / kWave;  // 16-byte pieces per lane of an input tile
    constexpr int OUT_PIECES = 32 * OUTW / 4 / kWave;
    static_assert(FOUT % 32 == 0 && FIN % 8 == 0, "staged kernel needs whole 32-column tiles");
    __shared__ float s_w[FIN * FOUT];
    __shared__ __attribute__((aligned(16))) float s_tile[kWavesPerBlock][32 * LDT];

    const int tid = threadIdx.x;
    for (int idx = tid; idx < FIN * FOUT; idx += kThreads) s_w[idx] = w[wt ? (idx % FOUT) * FIN + idx / FOUT : idx];
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int i = lane & 31, hh = lane >> 5;
    float *tile_lds = s_tile[wave];
    const int64_t stride = (int64_t)gridDim.x * kWavesPerBlock;
    const int64_t first = (int64_t)blockIdx.x * kWavesPerBlock + wave;
    const int64_t iters = (n_tiles - (int64_t)blockIdx.x * kWavesPerBlock + stride - 1) / stride;   // same for the whole block

    floatx4 in_next[IN_PIECES];
    auto fetch = [&](int64_t t) {
#pragma unroll
        for (int q = 0; q < IN_PIECES; ++q) {
            const int64_t piece = t * (32 * FIN / 4) + q * kWave + lane;      // 16-byte pieces from the start of X
            in_next[q] = (t < n_tiles && piece * 4 < n * FIN) ? __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(x) + piece)
                                                               : floatx4{0.f, 0.f, 0.f, 0.f};
        }
    };
    fetch(first);
    __syncthreads();
    for (int64_t it = 0; it < iters; ++it) {
        const int64_t tile = first + it * stride;
        // ---- input tile: registers -> LDS (padded rows)
#pragma unroll
        for (int q = 0; q < IN_PIECES; ++q) {
            const int e = (q * kWave + lane) * 4;                             // float index inside the tile
            *reinterpret_cast<floatx4 *>(&tile_lds[(e / FIN) * LDT + e % FIN]) = in_next[q];
        }
        fetch(tile + stride);
        wave_lds_sync();
        floatx4 a[KH / 4];
#pragma unroll
        for (int q = 0; q < KH / 4; ++q) a[q] = *reinterpret_cast<const floatx4 *>(&tile_lds[i * LDT + hh * KH + q * 4]);
        const int64_t row = tile * 32 + i;
        const float scale = (row_scale && tile < n_tiles && row < n) ? row_scale[row] : 1.0f;
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
                const float wv = s_w[(hh * KH + s) * FOUT + jt * 32 + i];
                acc[jt] = __builtin_amdgcn_mfma_f32_32x32x2f32(wv, xv, acc[jt], 0, 0, 0);   // (X W)^T tile
            }
        }
        wave_lds_sync();                                                      // every lane has its operands
        // ---- result tile: accumulators -> LDS -> whole lines
#pragma unroll
        for (int jt = 0; jt < NT; ++jt)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                *reinterpret_cast<floatx4 *>(&tile_lds[i * LDT + ROFF + jt * 32 + 8 * g + 4 * hh]) =
                    floatx4{acc[jt][4 * g] * scale, acc[jt][4 * g + 1] * scale, acc[jt][4 * g + 2] * scale,
                            acc[jt][4 * g + 3] * scale};
        wave_lds_sync();
        if (tile < n_tiles) {
#pragma unroll
            for (int q = 0; q < OUT_PIECES; ++q) {
                const int e = (q * kWave + lane) * 4;
                const int64_t piece = tile * (32 * OUTW / 4) + q * kWave + lane;
                if (piece * 4 < n * OUTW) {
                    floatx4 v = *reinterpret_cast<const floatx4 *>(&tile_lds[(e / OUTW) * LDT + e % OUTW]);
                    if (CONCAT) v = floatx4{fmaxf(v[0], 0.0f), fmaxf(v[1], 0.0f), fmaxf(v[2], 0.0f), fmaxf(v[3], 0.0f)};
                    __builtin_nontemporal_store(v, reinterpret_cast<floatx4 *>(h) + piece);   // whole lines, read by a later kernel: 4 % faster than plain stores
                }
            }
        }
        wave_lds_sync();                                                      // the tile buffer is reused
    }
}

template <int FIN, int FOUT>
__global__ __launch_bounds__(kThreads) void xw_bf16_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ w,
                                                           const float *__restrict__ row_scale, uint16_t *__restrict__ h,
                                                           int64_t n, int64_t n_tiles, int wt) {
    constexpr int NT = (FOUT + 31) / 32;
    constexpr int JG = NT > 2 ? 2 : NT;    // column tiles accumulated at a time (bounds the live accumulators)
    constexpr int KH = FIN / 2;            // bf16 values owned by one lane
    constexpr int KS = KH / 8;             // MFMA steps of depth 16 (8 per lane half)
    constexpr int LDW = FIN + 8;           // padded row of W^T in LDS, keeps 16-byte reads conflict-free
    __shared__ __attribute__((aligned(16))) uint16_t s_wt[NT * 32 * LDW];   // W transposed: [column][k]

    const int tid = threadIdx.x;
    for (int idx = tid; idx < FIN * NT * 32; idx += kThreads) {
        int k = idx / (NT * 32), j = idx % (NT * 32);
        s_wt[j * LDW + k] = j < FOUT ? w[wt ? j * FIN + k : k * FOUT + j] : (uint16_t)0;
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
        fetch(tile + stride);              // the next tile's rows travel while this one is multiplied
        const int64_t row = tile * 32 + i;
#pragma unroll
        for (int j0 = 0; j0 < NT; j0 += JG) {
            floatx16 acc[JG];
#pragma unroll
            for (int jj = 0; jj < JG; ++jj)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[jj][v] = 0.0f;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
#pragma unroll
                for (int jj = 0; jj < JG; ++jj) {
                    const bf16x8 wv = *reinterpret_cast<const bf16x8 *>(&s_wt[((j0 + jj) * 32 + i) * LDW + hh * KH + s * 8]);
                    acc[jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, a[s], acc[jj], 0, 0, 0);   // (X W)^T tile
                }
            }
            if (row < n) {
#pragma unroll
                for (int jj = 0; jj < JG; ++jj)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int col = (j0 + jj) * 32 + 8 * g + 4 * hh;
                        if (col < FOUT) {
                            const uint32_t lo = f32_to_bf16(acc[jj][4 * g] * scale) | (f32_to_bf16(acc[jj][4 * g + 1] * scale) << 16);
                            const uint32_t hi = f32_to_bf16(acc[jj][4 * g + 2] * scale) | (f32_to_bf16(acc[jj][4 * g + 3] * scale) << 16);
                            *reinterpret_cast<uint2 *>(h + row * FOUT + col) = make_uint2(lo, hi);
                        }
                    }
            }
            __builtin_amdgcn_sched_barrier(0);   // keep the column groups apart: their accumulators share registers
        }
    }
}

// bf16 with both widths at least 32: as the staged fp32 kernel, tiles pass through LDS so that every global
// access is a run of whole lines, and the transposed product leaves four consecutive columns per lane.
template <int FIN, int FOUT, bool CONCAT>
__global__ __launch_bounds__(kThreads) void xw_bf16_staged_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ w,
                                                                  const float *__restrict__ row_scale, uint16_t *__restrict__ h,
                                                                  int64_t n, int64_t n_tiles, int wt) {
    constexpr int NT = FOUT / 32;
    constexpr int JG = NT > 2 ? 2 : NT;              // column tiles accumulated at a time
    constexpr int KH = FIN / 2;
    constexpr int KS = KH / 8;
    constexpr int LDW = FIN + 8;                     // padded row of W^T (bf16 values)
    constexpr int FMAX = FIN > FOUT ? FIN : FOUT;
    constexpr int ROFF = CONCAT ? FIN : 0;           // as in the fp32 kernel
    constexpr int OUTW = CONCAT ? FIN + FOUT : FOUT;
    constexpr int LDT = (CONCAT ? FIN + FOUT : FMAX) + 8;   // padded tile row
    constexpr int IN_PIECES = 32 * FIN / 8 / kWave;  // 16-byte pieces per lane of an input tile
    constexpr int OUT_PIECES = 32 * OUTW / 8 / kWave;
    static_assert(FOUT % 32 == 0 && FIN % 32 == 0, "staged kernel needs whole 32-column tiles");
    __shared__ __attribute__((aligned(16))) uint16_t s_wt[FOUT * LDW];
    __shared__ __attribute__((aligned(16))) uint16_t s_tile[kWavesPerBlock][32 * LDT];

    const int tid = threadIdx.x;
    for (int idx = tid; idx < FIN * FOUT; idx += kThreads) {
        const int k = idx / FOUT, j = idx % FOUT;
        s_wt[j * LDW + k] = w[wt ? j * FIN + k : idx];
    }
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int i = lane & 31, hh = lane >> 5;
    uint16_t *tile_lds = s_tile[wave];
    const int64_t stride = (int64_t)gridDim.x * kWavesPerBlock;
    const int64_t first = (int64_t)blockIdx.x * kWavesPerBlock + wave;
    const int64_t iters = (n_tiles - (int64_t)blockIdx.x * kWavesPerBlock + stride - 1) / stride;   // same for the whole block

    uintx4 in_next[IN_PIECES];
    auto fetch = [&](int64_t t) {
#pragma unroll
        for (int q = 0; q < IN_PIECES; ++q) {
            const int64_t piece = t * (32 * FIN / 8) + q * kWave + lane;      // 16-byte pieces from the start of X
            in_next[q] = (t < n_tiles && piece * 8 < n * FIN) ? __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(x) + piece)
                                                               : uintx4{0u, 0u, 0u, 0u};
        }
    };
    fetch(first);
    __syncthreads();
    for (int64_t it = 0; it < iters; ++it) {
        const int64_t tile = first + it * stride;
#pragma unroll
        for (int q = 0; q < IN_PIECES; ++q) {
            const int e = (q * kWave + lane) * 8;                             // bf16 index inside the tile
            *reinterpret_cast<uintx4 *>(&tile_lds[(e / FIN) * LDT + e % FIN]) = in_next[q];
        }
        fetch(tile + stride);
        wave_lds_sync();
        bf16x8 a[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) a[s] = *reinterpret_cast<const bf16x8 *>(&tile_lds[i * LDT + hh * KH + s * 8]);
        const int64_t row = tile * 32 + i;
        const float scale = (row_scale && tile < n_tiles && row < n) ? row_scale[row] : 1.0f;
        wave_lds_sync();                                                      // every lane has its operands
#pragma unroll
        for (int j0 = 0; j0 < NT; j0 += JG) {
            floatx16 acc[JG];
#pragma unroll
            for (int jj = 0; jj < JG; ++jj)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[jj][v] = 0.0f;
#pragma unroll
            for (int s = 0; s < KS; ++s)
#pragma unroll
                for (int jj = 0; jj < JG; ++jj) {
                    const bf16x8 wv = *reinterpret_cast<const bf16x8 *>(&s_wt[((j0 + jj) * 32 + i) * LDW + hh * KH + s * 8]);
                    acc[jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, a[s], acc[jj], 0, 0, 0);   // (X W)^T tile
                }
#pragma unroll
            for (int jj = 0; jj < JG; ++jj)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const uint32_t lo = f32_to_bf16(acc[jj][4 * g] * scale) | (f32_to_bf16(acc[jj][4 * g + 1] * scale) << 16);
                    const uint32_t hi = f32_to_bf16(acc[jj][4 * g + 2] * scale) | (f32_to_bf16(acc[jj][4 * g + 3] * scale) << 16);
                    *reinterpret_cast<uint2 *>(&tile_lds[i * LDT + ROFF + (j0 + jj) * 32 + 8 * g + 4 * hh]) = make_uint2(lo, hi);
                }
            __builtin_amdgcn_sched_barrier(0);   // keep the column groups apart: their accumulators share registers
        }
        wave_lds_sync();
        if (tile < n_tiles) {
#pragma unroll
            for (int q = 0; q < OUT_PIECES; ++q) {
                const int e = (q * kWave + lane) * 8;
                const int64_t piece = tile * (32 * OUTW / 8) + q * kWave + lane;
                if (piece * 8 < n * OUTW) {
                    uintx4 v = *reinterpret_cast<const uintx4 *>(&tile_lds[(e / OUTW) * LDT + e % OUTW]);
                    if (CONCAT) {      // a bf16 with its sign bit set becomes zero (a negative zero too)
#pragma unroll
                        for (int c = 0; c < 4; ++c) v[c] = ((v[c] & 0x8000u) ? 0u : (v[c] & 0xffffu)) | ((v[c] & 0x80000000u) ? 0u : (v[c] & 0xffff0000u));
                    }
                    __builtin_nontemporal_store(v, reinterpret_cast<uintx4 *>(h) + piece);
                }
            }
        }
        wave_lds_sync();                                                      // the tile buffer is reused
    }
}

// Grid.  A large W wants a persistent launch: as many workgroups as the device holds at once, so that W is staged
// once per resident workgroup and every wavefront walks many row tiles.  A small W (up to 8 KB) is cheap to stage
// again, and then many short-lived workgroups stream faster than few long-lived ones (measured: 32 -> 32 fp32 on 2^24
// rows 0.83 -> 0.75 ms with one tile per wavefront): a wavefront then takes just enough tiles to move about 8 KB
// and to keep the staging of W a small share of its traffic.
template <int FIN, int FOUT>
int launch(const void *x, const void *w, int wt, const float *row_scale, void *h, int64_t n, dgnn_dtype dt, hipStream_t s) {
    const int64_t n_tiles = (n + 31) / 32;
    const int64_t needed = (n_tiles + kWavesPerBlock - 1) / kWavesPerBlock;
    const int64_t elem = dt == DGNN_F32 ? 4 : 2;
    const int64_t w_bytes = (int64_t)FIN * FOUT * elem, tile_bytes = 32 * (int64_t)(FIN + FOUT) * elem;
    const int64_t tiles_per_wave = w_bytes <= 4096 ? std::max<int64_t>(1, 8192 / tile_bytes) : w_bytes <= 8192 ? 4 : 0;
    auto grid = [&](auto kernel) {
        const int64_t resident = resident_workgroups(kernel, kThreads, 1024);
        const int64_t many = tiles_per_wave > 0 ? (needed + tiles_per_wave - 1) / tiles_per_wave : 0;
        return dim3((unsigned)(many >= 4 * resident ? many : std::min(needed, resident)));
    };
    if (dt == DGNN_F32) {
        if constexpr (FIN <= 64 && FOUT <= 64 && FOUT % 32 == 0)   // both tiles and W fit in LDS
            hipLaunchKernelGGL((xw_f32_staged_kernel<FIN, FOUT, false>), grid(xw_f32_staged_kernel<FIN, FOUT, false>), dim3(kThreads), 0, s,
                               static_cast<const float *>(x), static_cast<const float *>(w), row_scale, static_cast<float *>(h), n, n_tiles, wt);
        else
            hipLaunchKernelGGL((xw_f32_kernel<FIN, FOUT>), grid(xw_f32_kernel<FIN, FOUT>), dim3(kThreads), 0, s,
                               static_cast<const float *>(x), static_cast<const float *>(w), row_scale, static_cast<float *>(h), n, n_tiles, wt);
    } else {
        if constexpr (FIN % 32 == 0 && FOUT % 32 == 0)
            hipLaunchKernelGGL((xw_bf16_staged_kernel<FIN, FOUT, false>), grid(xw_bf16_staged_kernel<FIN, FOUT, false>), dim3(kThreads), 0, s,
                               static_cast<const uint16_t *>(x), static_cast<const uint16_t *>(w), row_scale,
                               static_cast<uint16_t *>(h), n, n_tiles, wt);
        else
            hipLaunchKernelGGL((xw_bf16_kernel<FIN, FOUT>), grid(xw_bf16_kernel<FIN, FOUT>), dim3(kThreads), 0, s,
                               static_cast<const uint16_t *>(x), static_cast<const uint16_t *>(w), row_scale,
                               static_cast<uint16_t *>(h), n, n_tiles, wt);
    }
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

// out = relu([x | x W]) where both tiles of a wavefront and W fit in LDS together; other width pairs are refused.
template <int FIN, int FOUT>
int launch_concat(const void *x, const void *w, void *out, int64_t n, dgnn_dtype dt, hipStream_t s) {
    const int64_t n_tiles = (n + 31) / 32;
    const int64_t needed = (n_tiles + kWavesPerBlock - 1) / kWavesPerBlock;
    const int64_t elem = dt == DGNN_F32 ? 4 : 2;
    const int64_t w_bytes = (int64_t)FIN * FOUT * elem, tile_bytes = 32 * (int64_t)(2 * FIN + FOUT) * elem;
    const int64_t tiles_per_wave = w_bytes <= 4096 ? std::max<int64_t>(1, 8192 / tile_bytes) : w_bytes <= 8192 ? 4 : 0;
    auto grid = [&](auto kernel) {      // as in launch(): short-lived workgroups when W is cheap to stage again
        const int64_t resident = resident_workgroups(kernel, kThreads, 1024);
        const int64_t many = tiles_per_wave > 0 ? (needed + tiles_per_wave - 1) / tiles_per_wave : 0;
        return dim3((unsigned)(many >= 4 * resident ? many : std::min(needed, resident)));
    };
    if (dt == DGNN_F32) {
        if constexpr (FIN <= 64 && FOUT <= 64 && FOUT % 32 == 0)
            hipLaunchKernelGGL((xw_f32_staged_kernel<FIN, FOUT, true>), grid(xw_f32_staged_kernel<FIN, FOUT, true>), dim3(kThreads), 0, s,
                               static_cast<const float *>(x), static_cast<const float *>(w), nullptr, static_cast<float *>(out), n, n_tiles, 0);
        else
            return DGNN_ERR_SHAPE;
    } else {
        if constexpr (FIN % 32 == 0 && FOUT % 32 == 0 && FIN + FOUT <= 128)
            hipLaunchKernelGGL((xw_bf16_staged_kernel<FIN, FOUT, true>), grid(xw_bf16_staged_kernel<FIN, FOUT, true>), dim3(kThreads), 0, s,
                               static_cast<const uint16_t *>(x), static_cast<const uint16_t *>(w), nullptr, static_cast<uint16_t *>(out), n,
                               n_tiles, 0);
        else
            return DGNN_ERR_SHAPE;
    }
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

template <int FIN>
int launch_concat_out(int32_t f_out, const void *x, const void *w, void *out, int64_t n, dgnn_dtype dt, hipStream_t s) {
    switch (f_out) {
        case 32: return launch_concat<FIN, 32>(x, w, out, n, dt, s);
        case 64: return launch_concat<FIN, 64>(x, w, out, n, dt, s);
        default: return DGNN_ERR_SHAPE;
    }
}

template <int FIN>
int launch_out(int32_t f_out, const void *x, const void *w, int wt, const float *row_scale, void *h, int64_t n,
               dgnn_dtype dt, hipStream_t s) {
    switch (f_out) {
        case 16: return launch<FIN, 16>(x, w, wt, row_scale, h, n, dt, s);
        case 32: return launch<FIN, 32>(x, w, wt, row_scale, h, n, dt, s);
        case 64: return launch<FIN, 64>(x, w, wt, row_scale, h, n, dt, s);
        case 128: return launch<FIN, 128>(x, w, wt, row_scale, h, n, dt, s);
        default: return DGNN_ERR_SHAPE;
    }
}

}  // namespace

namespace {

int transform(const void *x, int64_t n, int32_t f_in, const void *w, int wt, int32_t f_out, const float *row_scale,
              void *h, dgnn_dtype dt, void *stream) {
    if (!x || !w || !h) return DGNN_ERR_NULL;
    if (n <= 0 || !supported_width(f_in) || !supported_width(f_out)) return DGNN_ERR_SHAPE;
    if (dt != DGNN_F32 && dt != DGNN_BF16) return DGNN_ERR_SHAPE;
    if (!fits_index(n)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(x) || !aligned16(h)) return DGNN_ERR_ALIGN;
    if (x == h) return DGNN_ERR_ALIAS;
    hipStream_t s = (hipStream_t)stream;
    switch (f_in) {
        case 16: return launch_out<16>(f_out, x, w, wt, row_scale, h, n, dt, s);
        case 32: return launch_out<32>(f_out, x, w, wt, row_scale, h, n, dt, s);
        case 64: return launch_out<64>(f_out, x, w, wt, row_scale, h, n, dt, s);
        case 128: return launch_out<128>(f_out, x, w, wt, row_scale, h, n, dt, s);
        default: return DGNN_ERR_SHAPE;
    }
}

}  // namespace

extern "C" int dgnn_feature_transform(const void *x, int64_t n, int32_t f_in, const void *w, int32_t f_out,
                                      const float *row_scale, void *h, dgnn_dtype dt, void *stream) {
    return transform(x, n, f_in, w, 0, f_out, row_scale, h, dt, stream);
}

// dX = G W^T: the same product with W read transposed while it is parked in LDS; the contraction runs over
// the columns of W, so the kernel's inner width is f_out and its outer width f_in.
extern "C" int dgnn_input_grad(const void *g, int64_t n, int32_t f_out, const void *w, int32_t f_in,
                               const float *row_scale, void *dx, dgnn_dtype dt, void *stream) {
    return transform(g, n, f_out, w, 1, f_in, row_scale, dx, dt, stream);
}

// Y = relu([X | X W]): the dense transform with the skip connection of the CD-GCN layer's GCN operation (Section
// "CD-GCN") and its ReLU folded into the kernel that forms X W, so that X W itself never travels.
extern "C" int dgnn_transform_concat_relu(const void *x, int64_t n, int32_t f_in, const void *w, int32_t f_out, void *out,
                                          dgnn_dtype dt, void *stream) {
    if (!x || !w || !out) return DGNN_ERR_NULL;
    if (n <= 0 || !supported_width(f_in) || !supported_width(f_out)) return DGNN_ERR_SHAPE;
    if (dt != DGNN_F32 && dt != DGNN_BF16) return DGNN_ERR_SHAPE;
    if (!fits_index(n)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(x) || !aligned16(out)) return DGNN_ERR_ALIGN;
    if (x == out) return DGNN_ERR_ALIAS;
    hipStream_t s = (hipStream_t)stream;
    switch (f_in) {
        case 16: return launch_concat_out<16>(f_out, x, w, out, n, dt, s);
        case 32: return launch_concat_out<32>(f_out, x, w, out, n, dt, s);
        case 64: return launch_concat_out<64>(f_out, x, w, out, n, dt, s);
        default: return DGNN_ERR_SHAPE;
    }
}
