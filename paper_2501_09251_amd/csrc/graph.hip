// Graph of the sparsity pattern for the reordering (paper Section 3.2): one vertex per
// row/column index, an undirected unit-weight edge {i,j}, i != j, wherever A_ij or A_ji is
// stored.  Built on the GPU: both directions of every off-diagonal entry become 64-bit keys
// (i, j), a radix sort brings duplicates together, run heads are the directed edges, and a
// binary search per vertex gives the row pointers.  The result stays in device memory for the
// dendrogram step; copy_graph_to_host brings it to pinned host memory for the host form of
// that step.
#include "device_util.h"

namespace accspmm {
namespace {

using namespace detail;

// one wavefront per row
__global__ __launch_bounds__(256) void make_edge_keys_kernel(int64_t M, const int32_t* __restrict__ rowptr,
                                                             const int32_t* __restrict__ colidx, int32_t vbits,
                                                             uint64_t* __restrict__ keys) {
    int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= M) return;
    const int lane = threadIdx.x & 63;
    const int32_t b = rowptr[i], e = rowptr[i + 1];
    const uint64_t dropped = (uint64_t)1 << (2 * vbits);  // sorts after every real key
    for (int32_t p = b + lane; p < e; p += 64) {
        const uint64_t j = (uint32_t)colidx[p];
        const bool loop = j == (uint64_t)i;
        keys[2 * (int64_t)p] = loop ? dropped : (((uint64_t)i << vbits) | j);
        keys[2 * (int64_t)p + 1] = loop ? dropped : ((j << vbits) | (uint64_t)i);
    }
}

// distinct real keys -> neighbour list
__global__ void compact_edges_kernel(int64_t n, const uint64_t* __restrict__ sorted, const int32_t* __restrict__ head,
                                     const int32_t* __restrict__ upos, uint64_t dropped, uint64_t vmask,
                                     int32_t* __restrict__ adj) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < n && head[k] && sorted[k] != dropped) adj[upos[k]] = (int32_t)(sorted[k] & vmask);
}

// gptr[i] = number of sorted distinct keys below (i, 0), i = 0..M
__global__ void vertex_starts_kernel(int64_t M, int64_t n, const uint64_t* __restrict__ sorted,
                                     const int32_t* __restrict__ head_excl, int32_t vbits, int64_t* __restrict__ gptr) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > M) return;
    const uint64_t key = (uint64_t)i << vbits;
    int64_t lo = 0, len = n;  // first sorted position with key >= (i, 0)
    while (len > 0) {
        int64_t half = len >> 1;
        if (sorted[lo + half] < key) { lo += half + 1; len -= half + 1; } else len = half;
    }
    gptr[i] = head_excl[lo];  // distinct keys before that position (head_excl has n+1 entries)
}

}  // namespace

HostGraph::~HostGraph() {
    if (ptr) (void)hipHostFree(ptr);
    if (adj) (void)hipHostFree(adj);
}

void build_graph_on_device(int64_t M, int64_t nnz, const int32_t* d_rowptr, const int32_t* d_colidx, DeviceGraph& g) {
    g.M = M;
    g.two_m = 0;
    g.ptr.alloc(M + 1);
    if (nnz == 0) {
        ACC_HIP(hipMemset(g.ptr.p, 0, sizeof(int64_t) * (M + 1)));
        return;
    }
    const int vbits = bits_for(M);
    const int64_t n = 2 * nnz;
    const uint64_t dropped = (uint64_t)1 << (2 * vbits);
    Scratch tmp;
    DevBuf<uint64_t> keys, sorted;
    keys.alloc(n);
    sorted.alloc(n);
    hipLaunchKernelGGL(make_edge_keys_kernel, dim3(blocks_for(M, 4)), dim3(256), 0, 0, M, d_rowptr, d_colidx, vbits, keys.p);
    sort_keys_u64(tmp, keys.p, sorted.p, (size_t)n, (unsigned)(2 * vbits + 1));
    keys.release();
    DevBuf<int32_t> head, head_excl;
    head.alloc(n + 1);
    head_excl.alloc(n + 1);
    ACC_HIP(hipMemset(head.p + n, 0, sizeof(int32_t)));
    hipLaunchKernelGGL(mark_heads_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, 0, n, sorted.p, head.p);
    exclusive_scan_i32(tmp, head.p, head_excl.p, n + 1);
    // row pointers; ptr[M] counts the distinct real keys (the dropped key, if any, sorts last)
    hipLaunchKernelGGL(vertex_starts_kernel, dim3(blocks_for(M + 1, 256)), dim3(256), 0, 0, M, n, sorted.p, head_excl.p,
                       vbits, g.ptr.p);
    ACC_HIP(hipMemcpy(&g.two_m, g.ptr.p + M, sizeof(int64_t), hipMemcpyDeviceToHost));
    if (g.two_m > 0) {
        g.adj.alloc(g.two_m);
        hipLaunchKernelGGL(compact_edges_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, 0, n, sorted.p, head.p, head_excl.p,
                           dropped, ((uint64_t)1 << vbits) - 1, g.adj.p);
        ACC_HIP(hipGetLastError());
        ACC_HIP(hipDeviceSynchronize());
    }
}

void copy_graph_to_host(const DeviceGraph& d, HostGraph& g) {
    g.M = d.M;
    ACC_HIP(hipHostMalloc((void**)&g.ptr, sizeof(int64_t) * (d.M + 1), hipHostMallocDefault));
    ACC_HIP(hipMemcpy(g.ptr, d.ptr.p, sizeof(int64_t) * (d.M + 1), hipMemcpyDeviceToHost));
    if (d.two_m > 0) {
        ACC_HIP(hipHostMalloc((void**)&g.adj, sizeof(int32_t) * d.two_m, hipHostMallocDefault));
        ACC_HIP(hipMemcpy(g.adj, d.adj.p, sizeof(int32_t) * d.two_m, hipMemcpyDeviceToHost));
    }
}

}  // namespace accspmm
