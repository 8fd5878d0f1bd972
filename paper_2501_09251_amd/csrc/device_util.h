// Small device-side helpers shared by the plan's HIP translation units.
#pragma once
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_scan.hpp>

#include "internal.h"

namespace accspmm {
namespace detail {

struct Scratch {  // rocPRIM temporary storage, grown on demand
    DevBuf<char> buf;
    void* get(size_t bytes) {
        if (bytes > buf.n) buf.alloc(bytes);
        return buf.p;
    }
};

inline void exclusive_scan_i32(Scratch& tmp, const int32_t* in, int32_t* out, size_t n) {
    size_t bytes = 0;
    ACC_HIP(rocprim::exclusive_scan(nullptr, bytes, in, out, 0, n, rocprim::plus<int32_t>()));
    ACC_HIP(rocprim::exclusive_scan(tmp.get(bytes), bytes, in, out, 0, n, rocprim::plus<int32_t>()));
}

inline void sort_keys_u64(Scratch& tmp, uint64_t* in, uint64_t* out, size_t n, unsigned end_bit) {
    size_t bytes = 0;
    ACC_HIP(rocprim::radix_sort_keys(nullptr, bytes, in, out, n, 0u, end_bit));
    ACC_HIP(rocprim::radix_sort_keys(tmp.get(bytes), bytes, in, out, n, 0u, end_bit));
}

inline unsigned blocks_for(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

inline int bits_for(int64_t n) {  // bits needed to hold values in [0, n)
    int b = 1;
    while (((int64_t)1 << b) < n) ++b;
    return b;
}

// head[i] = 1 where a run of equal keys starts
[[maybe_unused]] static __global__ void mark_heads_kernel(int64_t n, const uint64_t* __restrict__ sorted, int32_t* __restrict__ head) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) head[i] = (i == 0 || sorted[i] != sorted[i - 1]) ? 1 : 0;
}

}  // namespace detail
}  // namespace accspmm
