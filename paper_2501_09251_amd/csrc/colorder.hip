// Column order of A = row order of B (the paper's Section 4.3.1 and its conclusion name
// column reordering of A with the matching row reordering of B as the next step after row
// reordering; the order itself is this library's choice).
//
// The order groups columns by how often they are used: class(c) = floor(log2(entries in
// column c)), classes in descending order, the original ids ascending inside a class, unused
// columns last.  The rows of B that many row windows gather (the hubs of a power-law graph)
// then sit next to each other at the start of B, whatever labels the input gave them, and
// inputs whose columns all have similar counts (meshes) keep their order.  Why it matters:
// on an R-MAT graph with unscrambled labels the hubs are the ids with few set bits, their
// rows of B lie at large power-of-two strides, and gathering them collides in the memory
// system; relabelling removed a quarter of the kernel time at 2^23 columns.
//
// Two ways to use the order.  The caller keeps B in it (all of SparseAToB in plan ids).  Or B
// stays in the caller's order and only the first n_hot rows of the order, which carry most of
// the gathers, are copied together before each execute; SparseAToB then names either a row of
// that copy or a row of B in place.
#include "device_util.h"

namespace accspmm {
namespace {

using detail::blocks_for;

__global__ void count_columns_kernel(int64_t nnz, const int32_t* __restrict__ colidx, int32_t* __restrict__ count) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nnz) atomicAdd(count + colidx[i], 1);
}

// key = 31 - floor(log2(count)) for used columns (so that ascending keys are descending
// classes), 32 for unused ones; value = the column id
__global__ void class_keys_kernel(int64_t K, const int32_t* __restrict__ count, uint32_t* __restrict__ key,
                                  int32_t* __restrict__ id) {
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= K) return;
    const int32_t n = count[c];
    key[c] = n > 0 ? (uint32_t)__builtin_clz((uint32_t)n) : 32u;
    id[c] = (int32_t)c;
}

__global__ void invert_kernel(int64_t K, const int32_t* __restrict__ order, int32_t* __restrict__ rank) {
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j < K) rank[order[j]] = (int32_t)j;
}

__global__ void remap_kernel(int64_t nnz, const int32_t* __restrict__ colidx, const int32_t* __restrict__ rank,
                             int32_t* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nnz) out[i] = rank[colidx[i]];
}

// Entries of SparseAToB in plan column ids -> what the tile kernel reads when B stays in the
// caller's order: plan column r < n_hot becomes ~r (row r of the gathered hot rows), the others
// become their input column order[r] (a row of B in place).
// `plain` (optional) gets the input column of every entry, for reading all of B in place.
__global__ void hot_cold_entries_kernel(int64_t n, int32_t* __restrict__ a2b, const int32_t* __restrict__ order,
                                        int32_t n_hot, int32_t* __restrict__ plain) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t r = a2b[i];
    const int32_t input_col = order[r];
    a2b[i] = r < n_hot ? ~r : input_col;
    if (plain) plain[i] = input_col;
}

// dst row j = src row order[j] (gather) or dst row order[j] = src row j (scatter); rows of
// `units` elements of type T
template <class T>
__global__ __launch_bounds__(256) void permute_rows_kernel(int64_t rows, int64_t units, const int32_t* __restrict__ order,
                                                           const T* __restrict__ src, T* __restrict__ dst, int scatter) {
    const int64_t total = rows * units;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t j = i / units, u = i - j * units;
        const int64_t other = order[j];
        if (scatter) dst[other * units + u] = src[i];
        else dst[i] = src[other * units + u];
    }
}

}  // namespace

void column_order_on_device(int64_t K, int64_t nnz, const int32_t* d_colidx, DevBuf<int32_t>& d_order,
                            DevBuf<int32_t>& d_rank) {
    detail::Scratch tmp;
    DevBuf<int32_t> count, id;
    DevBuf<uint32_t> key, key_sorted;
    count.alloc(K);
    id.alloc(K);
    key.alloc(K);
    key_sorted.alloc(K);
    d_order.alloc(K);
    d_rank.alloc(K);
    ACC_HIP(hipMemset(count.p, 0, sizeof(int32_t) * K));
    if (nnz > 0)
        hipLaunchKernelGGL(count_columns_kernel, dim3(blocks_for(nnz, 256)), dim3(256), 0, 0, nnz, d_colidx, count.p);
    hipLaunchKernelGGL(class_keys_kernel, dim3(blocks_for(K, 256)), dim3(256), 0, 0, K, count.p, key.p, id.p);
    // radix sort is stable: ids stay ascending inside a class
    size_t bytes = 0;
    ACC_HIP(rocprim::radix_sort_pairs(nullptr, bytes, key.p, key_sorted.p, id.p, d_order.p, (size_t)K, 0u, 6u));
    ACC_HIP(rocprim::radix_sort_pairs(tmp.get(bytes), bytes, key.p, key_sorted.p, id.p, d_order.p, (size_t)K, 0u, 6u));
    hipLaunchKernelGGL(invert_kernel, dim3(blocks_for(K, 256)), dim3(256), 0, 0, K, d_order.p, d_rank.p);
    ACC_HIP(hipGetLastError());
    ACC_HIP(hipDeviceSynchronize());
}

void remap_columns_on_device(int64_t nnz, const int32_t* d_colidx, const int32_t* d_rank, int32_t* d_out) {
    if (nnz == 0) return;
    hipLaunchKernelGGL(remap_kernel, dim3(blocks_for(nnz, 256)), dim3(256), 0, 0, nnz, d_colidx, d_rank, d_out);
    ACC_HIP(hipGetLastError());
}

void hot_cold_entries_on_device(int64_t n, int32_t* d_a2b, const int32_t* d_order, int32_t n_hot, int32_t* d_plain) {
    if (n == 0) return;
    hipLaunchKernelGGL(hot_cold_entries_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, 0, n, d_a2b, d_order, n_hot,
                       d_plain);
    ACC_HIP(hipGetLastError());
    ACC_HIP(hipDeviceSynchronize());
}

void launch_permute_rows(const int32_t* d_order, int64_t rows, const void* src, void* dst, int64_t row_bytes, bool scatter,
                         hipStream_t stream) {
    if (rows == 0 || row_bytes == 0) return;
    const bool vec = row_bytes % 16 == 0 && ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) == 0;
    const int64_t units = vec ? row_bytes / 16 : row_bytes / 2;
    const unsigned blocks = (unsigned)std::min<int64_t>((rows * units + 255) / 256, 256 * 32);
    typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
    if (vec)
        hipLaunchKernelGGL(permute_rows_kernel<uintx4>, dim3(blocks), dim3(256), 0, stream, rows, units, d_order,
                           static_cast<const uintx4*>(src), static_cast<uintx4*>(dst), scatter ? 1 : 0);
    else
        hipLaunchKernelGGL(permute_rows_kernel<uint16_t>, dim3(blocks), dim3(256), 0, stream, rows, units, d_order,
                           static_cast<const uint16_t*>(src), static_cast<uint16_t*>(dst), scatter ? 1 : 0);
    ACC_HIP(hipGetLastError());
}

}  // namespace accspmm
