// Column layout of a sparse matrix from its row layout, on the device, once per matrix: for a
// caller that supplies CSR only.  A stable sort of the entries by column (row-major input, so the
// rows of every column come out ascending and repeated entries keep their order): the result is a
// function of the input alone, which is what keeps reruns bit-identical.  The sort itself is the
// library routine (rocPRIM's radix sort on the column index, the (row, value) pair as payload);
// this is set-up work, not part of an iteration.
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>

#include "sparse_internal.h"

namespace slaqglm {

namespace {

// keys[e] = column of entry e, vals[e] = (row << 32) | bits of the value.  One thread per entry;
// its row is the last r with row_ptr[r] <= e.
__global__ __launch_bounds__(256) void csc_expand_kernel(const long long *__restrict__ row_ptr, long long N,
                                                         const int *__restrict__ col_idx,
                                                         const float *__restrict__ row_val, long long nnz,
                                                         int *__restrict__ keys, unsigned long long *__restrict__ vals) {
    const long long e = blockIdx.x * 256LL + threadIdx.x;
    if (e >= nnz) return;
    long long lo = 0, hi = N - 1;
    while (lo < hi) {
        const long long mid = lo + (hi - lo + 1) / 2;
        if (row_ptr[mid] <= e) lo = mid; else hi = mid - 1;
    }
    keys[e] = col_idx[e];
    vals[e] = ((unsigned long long)lo << 32) | (unsigned long long)__float_as_uint(row_val[e]);
}

__global__ __launch_bounds__(256) void csc_unpack_kernel(const unsigned long long *__restrict__ vals, long long nnz,
                                                         int *__restrict__ row_idx, float *__restrict__ col_val) {
    const long long e = blockIdx.x * 256LL + threadIdx.x;
    if (e >= nnz) return;
    const unsigned long long v = vals[e];
    row_idx[e] = (int)(v >> 32);
    col_val[e] = __uint_as_float((unsigned)v);
}

// col_ptr[d] = first position whose (sorted) column is >= d, for d = 0 .. D
__global__ __launch_bounds__(256) void csc_colptr_kernel(const int *__restrict__ keys, long long nnz, long long D,
                                                         long long *__restrict__ col_ptr) {
    const long long d = blockIdx.x * 256LL + threadIdx.x;
    if (d > D) return;
    long long lo = 0, hi = nnz;                   // first p in [0, nnz] with keys[p] >= d
    while (lo < hi) {
        const long long mid = lo + (hi - lo) / 2;
        if ((long long)keys[mid] < d) lo = mid + 1; else hi = mid;
    }
    col_ptr[d] = lo;
}

}  // namespace

size_t sparse_csc_temp_bytes(long long nnz) { return ((size_t)64 << 20) + 2 * (size_t)(nnz > 0 ? nnz : 0); }

hipError_t launch_sparse_csc_build(const SparseArgs &a, const SparseCsc &c, hipStream_t st) {
    hipError_t e;
    if (a.nnz > 0) {
        const unsigned nb = (unsigned)((a.nnz + 255) / 256);
        hipLaunchKernelGGL(csc_expand_kernel, dim3(nb), dim3(256), 0, st, a.row_ptr, a.N, a.col_idx, a.row_val, a.nnz,
                           c.keys[0], c.vals[0]);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        rocprim::double_buffer<int> keys(c.keys[0], c.keys[1]);
        rocprim::double_buffer<unsigned long long> vals(c.vals[0], c.vals[1]);
        unsigned bits = 1;
        while (bits < 31 && (1LL << bits) < a.D) ++bits;
        size_t need = 0;
        if ((e = rocprim::radix_sort_pairs(nullptr, need, keys, vals, (size_t)a.nnz, 0u, bits, st)) != hipSuccess) return e;
        if (need > c.temp_bytes) return hipErrorOutOfMemory;
        if ((e = rocprim::radix_sort_pairs(c.temp, need, keys, vals, (size_t)a.nnz, 0u, bits, st)) != hipSuccess) return e;
        hipLaunchKernelGGL(csc_unpack_kernel, dim3(nb), dim3(256), 0, st, vals.current(), a.nnz, c.row_idx, c.col_val);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(csc_colptr_kernel, dim3((unsigned)((a.D + 1 + 255) / 256)), dim3(256), 0, st, keys.current(),
                           a.nnz, a.D, c.col_ptr);
        return hipGetLastError();
    }
    return hipMemsetAsync(c.col_ptr, 0, sizeof(long long) * (size_t)(a.D + 1), st);
}

}  // namespace slaqglm
