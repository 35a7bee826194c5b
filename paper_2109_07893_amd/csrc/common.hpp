// Internal helpers shared by the HIP sources of libdgnn (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>
#include <utility>
#include <vector>

#include "dgnn.h"

#define DGNN_RETURN_IF_LAUNCH_FAILED()                       \
    do {                                                     \
        if (hipGetLastError() != hipSuccess) return DGNN_ERR_HIP; \
    } while (0)

namespace dgnn {

constexpr int kWave = 64;   // wavefront width on CDNA4

inline bool fits_i32(int64_t v) { return v >= 0 && v <= 2147483647LL; }
// Row and entry counts: kernels form "index + a tile's worth" in int32 before comparing with the count, so the
// counts themselves stop 2^16 short of 2^31.
inline bool fits_index(int64_t v) { return v >= 0 && v <= 2147483647LL - 65536; }
inline bool supported_width(int32_t f) { return f == 16 || f == 32 || f == 64 || f == 128; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Workgroups of `threads` threads of `kernel` that the device holds at once (compute units x workgroups per unit):
// the grid of a kernel whose workgroups walk their share of the work in a loop.  Asked of the runtime once per
// kernel (keyed by the kernel's address: kernels of equal signature are different kernels) and remembered; `fallback`
// if the runtime cannot say.
template <typename K>
inline int64_t resident_workgroups(K kernel, int threads, int64_t fallback) {
    static std::mutex lock;
    static std::vector<std::pair<const void *, int64_t>> known;
    const void *key = reinterpret_cast<const void *>(kernel);
    std::lock_guard<std::mutex> guard(lock);
    for (const auto &kv : known)
        if (kv.first == key) return kv.second;
    int dev = 0, cus = 0, per_cu = 0;
    int64_t value = fallback;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) == hipSuccess && cus > 0 && per_cu > 0)
        value = (int64_t)cus * per_cu;
    else
        (void)hipGetLastError();
    known.emplace_back(key, value);
    return value;
}

// First index in [lo, hi) whose element is >= key (array ascending).
__device__ __forceinline__ int lower_bound(const int32_t *__restrict__ a, int lo, int hi, int32_t key) {
    while (lo < hi) {
        int mid = lo + ((hi - lo) >> 1);
        if (a[mid] < key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// Largest r in [0, n) with rowptr[r] <= key (-1 if there is none), for a non-decreasing rowptr.
// A 64-ary search done by one whole wavefront: every lane of the wavefront must call it with the
// same arguments; each round probes 64 evenly spaced entries at once, so 2^24 rows take four
// dependent loads instead of twenty-four.
__device__ __forceinline__ int wave_find_row(const int32_t *__restrict__ rowptr, int n, int key, int lane) {
    int lo = 0, hi = n;   // the first index whose entry exceeds key lies in [lo, hi]
    while (hi > lo) {
        const int step = (hi - lo + kWave - 1) / kWave;
        const int idx = lo + lane * step;
        const bool le = idx < hi && rowptr[idx] <= key;
        const int m = __popcll(__ballot(le));   // monotone: exactly lanes 0 .. m-1 hold entries <= key
        if (m == 0) { hi = lo; break; }
        const int nlo = lo + (m - 1) * step + 1;
        hi = min(lo + m * step, hi);
        lo = nlo;
    }
    return lo - 1;
}

// Orders the LDS traffic of ONE wavefront: what its lanes have written to LDS before is visible to all of its
// lanes after.  No s_barrier: other wavefronts of the workgroup are not waited for, so wavefronts that work on
// private LDS tiles can drift apart (one loads while another multiplies).  The fences are of wavefront scope: the
// LDS serves one wavefront's accesses in the order it issued them, so nothing has to be waited for (a workgroup-scope
// fence drains the wavefront's LDS queue first); the fences only keep the compiler from moving LDS accesses across
// this point.  Loads from global memory that are in flight stay in flight either way.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Inclusive wavefront scans over 64 lanes.
__device__ __forceinline__ int wave_scan_add(int v, int lane) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        int o = __shfl_up(v, d, kWave);
        if (lane >= d) v += o;
    }
    return v;
}
__device__ __forceinline__ int wave_scan_max(int v, int lane) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        int o = __shfl_up(v, d, kWave);
        if (lane >= d) v = max(v, o);
    }
    return v;
}

// bfloat16 <-> float, round to nearest even on the way down.
__device__ __forceinline__ float bf16_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// ---- 16-byte pieces of feature rows: 4 fp32 or 8 bf16 values, unpacked to and packed from fp32 ------------
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

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

__device__ __forceinline__ float sigmoidf(float x) { return 1.0f / (1.0f + expf(-x)); }

}  // namespace dgnn
