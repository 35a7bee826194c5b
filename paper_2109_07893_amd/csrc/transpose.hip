// Transposed snapshots and transposed difference lists (Section "Gradient Checkpoint": gradients travel through a
// block in the reverse direction, and the adjoint of the aggregation A~ H is A~^T G).  For a directed dynamic graph
// the transposed snapshots form a dynamic graph of their own; what a caller has to prepare for it is A_1^T in the
// same canonical CSR form and every difference list re-sorted by (col, row) with rows and columns exchanged.  Both are
// the same operation: sort the stored pairs by (column, row).  The sort itself is the library's radix sort on 64-bit
// keys (the column above the row, as many bits each as an index below n needs); the kernels here form the keys and
// take the result apart.
// Input formatting, run once per block or list, not part of the per-timestep path.
#include <hip/hip_runtime.h>

#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>

#include "common.hpp"

namespace {

using namespace dgnn;

constexpr int kThreads = 256;
constexpr int kPerThread = 4;    // consecutive entries per thread: one row search, then the row pointers are walked

// key[e] = (colidx[e] << bits) | row of e
__global__ __launch_bounds__(kThreads) void csr_keys_kernel(int n, int nnz, int bits, const int32_t *__restrict__ rowptr,
                                                           const int32_t *__restrict__ colidx, uint64_t *__restrict__ keys) {
    const int64_t first = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * kPerThread;
    if (first >= nnz) return;
    // the row that holds entry `first`: the last one whose pointer is <= first
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = lo + ((hi - lo) >> 1);
        if (rowptr[mid + 1] <= first) lo = mid + 1; else hi = mid;
    }
    int row = lo, row_end = rowptr[min(row + 1, n)];
    const int last = (int)min(first + kPerThread, (int64_t)nnz);
    for (int e = (int)first; e < last; ++e) {
        while (e >= row_end && row < n - 1) row_end = rowptr[++row + 1];     // rows without entries are stepped over
        keys[e] = ((uint64_t)(uint32_t)colidx[e] << bits) | (uint32_t)row;
    }
}

// key[e] = (col[e] << bits) | row[e]
__global__ __launch_bounds__(kThreads) void coo_keys_kernel(int64_t m, int bits, const int32_t *__restrict__ row,
                                                           const int32_t *__restrict__ col, uint64_t *__restrict__ keys) {
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e < m) keys[e] = ((uint64_t)(uint32_t)col[e] << bits) | (uint32_t)row[e];
}

// sorted keys -> the column indices of the transposed snapshot (the low parts of the keys)
__global__ __launch_bounds__(kThreads) void csr_unpack_kernel(int nnz, int bits, const uint64_t *__restrict__ keys,
                                                             int32_t *__restrict__ colidx_t) {
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e < nnz) colidx_t[e] = (int32_t)(keys[e] & (((uint64_t)1 << bits) - 1));
}

// ... and its row pointers: row r of the transposed snapshot begins at the first key whose high part is >= r (one
// search per row, so that stretches of rows without entries cost no more than any other rows)
__global__ __launch_bounds__(kThreads) void csr_rowptr_kernel(int n, int nnz, int bits, const uint64_t *__restrict__ keys,
                                                             int32_t *__restrict__ rowptr_t) {
    const int64_t r = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (r > n) return;
    const uint64_t want = (uint64_t)r << bits;
    int lo = 0, hi = nnz;
    while (lo < hi) {
        const int mid = lo + ((hi - lo) >> 1);
        if (keys[mid] < want) lo = mid + 1; else hi = mid;
    }
    rowptr_t[r] = lo;
}

__global__ __launch_bounds__(kThreads) void coo_unpack_kernel(int64_t m, int bits, const uint64_t *__restrict__ keys,
                                                             int32_t *__restrict__ row_t, int32_t *__restrict__ col_t) {
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e >= m) return;
    const uint64_t k = keys[e];
    row_t[e] = (int32_t)(k >> bits);
    col_t[e] = (int32_t)(k & (((uint64_t)1 << bits) - 1));
}

// Bits of the key that can differ: both words hold indices below n.
int index_bits(int64_t n) {
    int b = 1;
    while (((int64_t)1 << b) < n) ++b;
    return b;
}

struct Layout {
    size_t keys_in, keys_out, sort_tmp, total;
};

// Workspace: two key arrays of `count` entries and whatever the sort asks for (asked of the library, which answers for
// the current device, with null storage).
int layout(int64_t count, int bits, bool with_values, Layout *L) {
    size_t tmp = 0;
    uint64_t *nk = nullptr;
    float *nv = nullptr;
    const unsigned int sz = (unsigned int)std::max<int64_t>(count, 1);
    hipError_t rc = with_values ? rocprim::radix_sort_pairs(nullptr, tmp, nk, nk, nv, nv, sz, 0, 2 * bits, (hipStream_t)0)
                                : rocprim::radix_sort_keys(nullptr, tmp, nk, nk, sz, 0, 2 * bits, (hipStream_t)0);
    if (rc != hipSuccess) {
        (void)hipGetLastError();
        return DGNN_ERR_HIP;
    }
    const size_t karr = round_up((size_t)std::max<int64_t>(count, 1) * sizeof(uint64_t), 256);
    L->keys_in = 0;
    L->keys_out = karr;
    L->sort_tmp = 2 * karr;
    L->total = 2 * karr + round_up(tmp, 256) + 256;
    return DGNN_OK;
}

int sort_keys(uint64_t *in, uint64_t *out, const float *val_in, float *val_out, int64_t count, int bits, void *tmp, size_t tmp_bytes,
              hipStream_t s) {
    const unsigned int sz = (unsigned int)count;
    hipError_t rc = val_in ? rocprim::radix_sort_pairs(tmp, tmp_bytes, in, out, val_in, val_out, sz, 0, 2 * bits, s)
                           : rocprim::radix_sort_keys(tmp, tmp_bytes, in, out, sz, 0, 2 * bits, s);
    if (rc != hipSuccess) (void)hipGetLastError();
    return rc == hipSuccess ? DGNN_OK : DGNN_ERR_HIP;
}

}  // namespace

extern "C" int dgnn_csr_transpose_workspace(int64_t n, int64_t nnz, int with_values, size_t *bytes) {
    if (!bytes) return DGNN_ERR_NULL;
    if (n <= 0 || nnz < 0) return DGNN_ERR_SHAPE;
    if (!fits_index(n + 1) || !fits_index(nnz)) return DGNN_ERR_OVERFLOW;
    Layout L;
    const int rc = layout(nnz, index_bits(n), with_values != 0, &L);
    if (rc != DGNN_OK) return rc;
    *bytes = L.total;
    return DGNN_OK;
}

extern "C" int dgnn_csr_transpose(int64_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *val,
                                  int32_t *rowptr_t, int32_t *colidx_t, float *val_t, void *ws, size_t ws_bytes, void *stream) {
    if (!rowptr || !rowptr_t || !ws) return DGNN_ERR_NULL;
    if (nnz > 0 && (!colidx || !colidx_t)) return DGNN_ERR_NULL;
    if ((val != nullptr) != (val_t != nullptr)) return DGNN_ERR_NULL;
    if (n <= 0 || nnz < 0) return DGNN_ERR_SHAPE;
    if (!fits_index(n + 1) || !fits_index(nnz)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(ws)) return DGNN_ERR_ALIGN;
    if (rowptr_t == rowptr || (nnz > 0 && colidx_t == colidx) || (val && val_t == val)) return DGNN_ERR_ALIAS;
    Layout L;
    const int bits = index_bits(n);
    int rc = layout(nnz, bits, val != nullptr, &L);
    if (rc != DGNN_OK) return rc;
    if (ws_bytes < L.total) return DGNN_ERR_CAPACITY;
    hipStream_t s = (hipStream_t)stream;
    char *base = static_cast<char *>(ws);
    uint64_t *keys_in = reinterpret_cast<uint64_t *>(base + L.keys_in), *keys_out = reinterpret_cast<uint64_t *>(base + L.keys_out);
    if (nnz > 0) {
        const int64_t threads = (nnz + kPerThread - 1) / kPerThread;
        hipLaunchKernelGGL(csr_keys_kernel, dim3((unsigned)((threads + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, (int)n, (int)nnz,
                           bits, rowptr, colidx, keys_in);
        DGNN_RETURN_IF_LAUNCH_FAILED();
        rc = sort_keys(keys_in, keys_out, val, val_t, nnz, bits, base + L.sort_tmp, L.total - L.sort_tmp, s);
        if (rc != DGNN_OK) return rc;
        hipLaunchKernelGGL(csr_unpack_kernel, dim3((unsigned)((nnz + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, (int)nnz, bits,
                           keys_out, colidx_t);
        DGNN_RETURN_IF_LAUNCH_FAILED();
    }
    hipLaunchKernelGGL(csr_rowptr_kernel, dim3((unsigned)((n + 1 + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, (int)n, (int)nnz, bits,
                       keys_out, rowptr_t);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}

extern "C" int dgnn_coo_transpose_workspace(int64_t n, int64_t m, size_t *bytes) {
    if (!bytes) return DGNN_ERR_NULL;
    if (n <= 0 || m < 0) return DGNN_ERR_SHAPE;
    if (!fits_index(n + 1) || !fits_index(m)) return DGNN_ERR_OVERFLOW;
    Layout L;
    const int rc = layout(m, index_bits(n), false, &L);
    if (rc != DGNN_OK) return rc;
    *bytes = L.total;
    return DGNN_OK;
}

extern "C" int dgnn_coo_transpose(int64_t n, int64_t m, const int32_t *row, const int32_t *col, int32_t *row_t, int32_t *col_t,
                                  void *ws, size_t ws_bytes, void *stream) {
    if (!ws) return DGNN_ERR_NULL;
    if (m > 0 && (!row || !col || !row_t || !col_t)) return DGNN_ERR_NULL;
    if (n <= 0 || m < 0) return DGNN_ERR_SHAPE;
    if (!fits_index(n + 1) || !fits_index(m)) return DGNN_ERR_OVERFLOW;
    if (!aligned16(ws)) return DGNN_ERR_ALIGN;
    Layout L;
    const int bits = index_bits(n);
    int rc = layout(m, bits, false, &L);
    if (rc != DGNN_OK) return rc;
    if (ws_bytes < L.total) return DGNN_ERR_CAPACITY;
    if (m == 0) return DGNN_OK;
    hipStream_t s = (hipStream_t)stream;
    char *base = static_cast<char *>(ws);
    uint64_t *keys_in = reinterpret_cast<uint64_t *>(base + L.keys_in), *keys_out = reinterpret_cast<uint64_t *>(base + L.keys_out);
    const unsigned grid = (unsigned)((m + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(coo_keys_kernel, dim3(grid), dim3(kThreads), 0, s, m, bits, row, col, keys_in);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    rc = sort_keys(keys_in, keys_out, nullptr, nullptr, m, bits, base + L.sort_tmp, L.total - L.sort_tmp, s);
    if (rc != DGNN_OK) return rc;
    hipLaunchKernelGGL(coo_unpack_kernel, dim3(grid), dim3(kThreads), 0, s, m, bits, keys_out, row_t, col_t);
    DGNN_RETURN_IF_LAUNCH_FAILED();
    return DGNN_OK;
}
