// CSR -> bitmap tile format on the GPU (paper Section 3.3: RowWindowOffset, TCOffset,
// SparseAToB, TCLocalBit and the values packed in bit order), for WH x TW tiles.
//
// Pipeline (every step is data-parallel and order-independent, so the result is
// deterministic):
//   1. lengths of the reordered rows -> exclusive scan -> reordered row pointers
//   2. one 64-bit key (window, column) per stored entry
//   3. radix sort of the keys; heads of equal runs are the distinct columns of each window
//   4. distinct columns per window (a binary search per window boundary) -> tiles per window
//      -> RowWindowOffset (scan)
//   5. SparseAToB: each window's distinct columns, the last tile padded with the last column
//   6. TCLocalBit: every entry finds its condensed column by binary search and sets its bit
//   7. TCOffset: scan of the tiles' popcounts
//   8. values: entry -> TCOffset[tile] + popcount(lower bits)
// The sort and the scans are rocPRIM device primitives; the rest are the kernels below.
#include "device_util.h"

namespace accspmm {
namespace {

using namespace detail;

__global__ void row_lengths_kernel(int64_t M, const int32_t* __restrict__ rowptr, const int32_t* __restrict__ perm,
                                   int32_t* __restrict__ len) {
    int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r < M) {
        int32_t i = perm[r];
        len[r] = rowptr[i + 1] - rowptr[i];
    }
}

// one wavefront per reordered row
__global__ __launch_bounds__(256) void make_keys_kernel(int64_t M, const int32_t* __restrict__ rowptr,
                                                        const int32_t* __restrict__ colidx,
                                                        const int32_t* __restrict__ perm,
                                                        const int32_t* __restrict__ new_rowptr, int32_t WH,
                                                        int32_t colbits, uint64_t* __restrict__ keys) {
    int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= M) return;
    const int lane = threadIdx.x & 63;
    const int32_t src = rowptr[perm[r]], dst = new_rowptr[r], len = new_rowptr[r + 1] - dst;
    const uint64_t hi = (uint64_t)(r / WH) << colbits;
    for (int32_t k = lane; k < len; k += 64) keys[dst + k] = hi | (uint32_t)colidx[src + k];
}

__global__ void compact_heads_kernel(int64_t n, const uint64_t* __restrict__ sorted, const int32_t* __restrict__ head,
                                     const int32_t* __restrict__ upos, uint64_t* __restrict__ uniq) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n && head[i]) uniq[upos[i]] = sorted[i];
}

// ustart[w] = first position in the sorted distinct keys whose window is >= w (w = 0..W)
__global__ void window_starts_kernel(int64_t W, int64_t n_unique, const uint64_t* __restrict__ uniq, int32_t colbits,
                                     int32_t* __restrict__ ustart) {
    int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (w > W) return;
    const uint64_t key = (uint64_t)w << colbits;
    int64_t lo = 0, n = n_unique;
    while (n > 0) {
        int64_t half = n >> 1;
        if (uniq[lo + half] < key) { lo += half + 1; n -= half + 1; } else n = half;
    }
    ustart[w] = (int32_t)lo;
}

__global__ void distinct_per_window_kernel(int64_t W, const int32_t* __restrict__ ustart, int32_t* __restrict__ dw) {
    int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (w < W) dw[w] = ustart[w + 1] - ustart[w];
}

__global__ void tiles_per_window_kernel(int64_t W, const int32_t* __restrict__ dw, int32_t TW, int32_t* __restrict__ tw) {
    int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (w < W) tw[w] = (dw[w] + TW - 1) / TW;
}

// one 64-thread block per window
__global__ __launch_bounds__(64) void fill_a2b_kernel(const int32_t* __restrict__ rwo, const int32_t* __restrict__ ustart,
                                                      const uint64_t* __restrict__ uniq, int32_t TW, uint64_t colmask,
                                                      int32_t* __restrict__ a2b) {
    const int64_t w = blockIdx.x;
    const int32_t t0 = rwo[w], nt = rwo[w + 1] - t0, u0 = ustart[w], d = ustart[w + 1] - u0;
    const int64_t total = (int64_t)nt * TW;
    for (int64_t e = threadIdx.x; e < total; e += 64) {
        int64_t k = e < d ? e : d - 1;
        a2b[(int64_t)t0 * TW + e] = (int32_t)(uniq[u0 + k] & colmask);
    }
}

// one wavefront per reordered row: set bits, remember (tile, bit) of every entry
__global__ __launch_bounds__(256) void set_bits_kernel(int64_t M, const int32_t* __restrict__ rowptr,
                                                       const int32_t* __restrict__ colidx,
                                                       const int32_t* __restrict__ perm,
                                                       const int32_t* __restrict__ new_rowptr,
                                                       const int32_t* __restrict__ rwo,
                                                       const int32_t* __restrict__ ustart,
                                                       const uint64_t* __restrict__ uniq, int32_t WH, int32_t TW,
                                                       int32_t NW, int32_t colbits, unsigned long long* __restrict__ bits,
                                                       int32_t* __restrict__ tile_of, uint16_t* __restrict__ bit_of) {
    int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= M) return;
    const int lane = threadIdx.x & 63;
    const int64_t w = r / WH;
    const int32_t rl = (int32_t)(r - w * WH);
    const int32_t src = rowptr[perm[r]], dst = new_rowptr[r], len = new_rowptr[r + 1] - dst;
    const int32_t u0 = ustart[w], d = ustart[w + 1] - u0, t0 = rwo[w];
    const uint64_t hi = (uint64_t)w << colbits;
    for (int32_t k = lane; k < len; k += 64) {
        const uint64_t key = hi | (uint32_t)colidx[src + k];
        int32_t lo = 0, n = d;  // first index with uniq[u0+idx] >= key (key is present)
        while (n > 0) {
            int32_t half = n >> 1;
            if (uniq[u0 + lo + half] < key) { lo += half + 1; n -= half + 1; } else n = half;
        }
        const int32_t g = t0 + lo / TW;
        const int32_t bit = rl * TW + lo % TW;
        atomicOr(&bits[(int64_t)g * NW + (bit >> 6)], 1ull << (bit & 63));
        tile_of[dst + k] = g;
        bit_of[dst + k] = (uint16_t)bit;
    }
}

__global__ void tile_popcount_kernel(int64_t T, const uint64_t* __restrict__ bits, int32_t NW, int32_t* __restrict__ cnt) {
    int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g < T) {
        int32_t c = 0;
        for (int k = 0; k < NW; ++k) c += __popcll(bits[g * NW + k]);
        cnt[g] = c;
    }
}

__global__ __launch_bounds__(256) void scatter_values_kernel(int64_t M, const int32_t* __restrict__ rowptr,
                                                             const uint16_t* __restrict__ vals,
                                                             const int32_t* __restrict__ perm,
                                                             const int32_t* __restrict__ new_rowptr,
                                                             const int32_t* __restrict__ tile_of,
                                                             const uint16_t* __restrict__ bit_of,
                                                             const uint64_t* __restrict__ bits, int32_t NW,
                                                             const int32_t* __restrict__ tco, uint16_t* __restrict__ packed,
                                                             int32_t* __restrict__ entry_of) {
    int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= M) return;
    const int lane = threadIdx.x & 63;
    const int32_t src = rowptr[perm[r]], dst = new_rowptr[r], len = new_rowptr[r + 1] - dst;
    for (int32_t k = lane; k < len; k += 64) {
        const int32_t g = tile_of[dst + k];
        const int32_t bit = bit_of[dst + k];
        const uint64_t* bm = bits + (int64_t)g * NW;
        int32_t rank = 0;
        for (int q = 0; q < (bit >> 6); ++q) rank += __popcll(bm[q]);
        rank += __popcll(bm[bit >> 6] & ((1ull << (bit & 63)) - 1ull));
        packed[tco[g] + rank] = vals[src + k];
        if (entry_of) entry_of[tco[g] + rank] = src + k;  // which CSR entry sits at this packed position
    }
}

}  // namespace

void encode_on_device(int64_t M, int64_t K, int64_t nnz, const int32_t* d_rowptr, const int32_t* d_colidx,
                      const uint16_t* d_vals, const int32_t* d_perm, int32_t WH, int32_t TW, DeviceFormat& out,
                      bool tiles_only, DevBuf<int32_t>* entry_of) {
    const int64_t W = (M + WH - 1) / WH;
    const int32_t NW = (WH * TW + 63) / 64;
    out.WH = WH; out.TW = TW; out.NW = NW; out.M = M; out.W = W; out.nnz = nnz; out.T = 0; out.sum_dw = 0;
    out.row_window_offset.alloc(W + 1);
    if (W == 0 || nnz == 0) {
        ACC_HIP(hipMemset(out.row_window_offset.p, 0, sizeof(int32_t) * (W + 1)));
        if (!tiles_only) {
            out.tc_offset.alloc(1);
            ACC_HIP(hipMemset(out.tc_offset.p, 0, sizeof(int32_t)));
            out.sparse_a_to_b.alloc(0);
            out.tc_local_bit.alloc(0);
            out.vals.alloc(16);
            ACC_HIP(hipMemset(out.vals.p, 0, 32));
        }
        return;
    }
    const int colbits = bits_for(K), winbits = bits_for(W);
    Scratch tmp;

    // 1. reordered row pointers
    DevBuf<int32_t> len, new_rowptr;
    len.alloc(M + 1);
    new_rowptr.alloc(M + 1);
    ACC_HIP(hipMemset(len.p, 0, sizeof(int32_t) * (M + 1)));
    hipLaunchKernelGGL(row_lengths_kernel, dim3(blocks_for(M, 256)), dim3(256), 0, 0, M, d_rowptr, d_perm, len.p);
    exclusive_scan_i32(tmp, len.p, new_rowptr.p, M + 1);
    len.release();

    // 2-3. keys, sort
    DevBuf<uint64_t> keys, sorted;
    keys.alloc(nnz);
    sorted.alloc(nnz);
    hipLaunchKernelGGL(make_keys_kernel, dim3(blocks_for(M, 4)), dim3(256), 0, 0, M, d_rowptr, d_colidx, d_perm,
                       new_rowptr.p, WH, colbits, keys.p);
    sort_keys_u64(tmp, keys.p, sorted.p, (size_t)nnz, (unsigned)(colbits + winbits));
    keys.release();

    // 4. distinct columns per window
    DevBuf<int32_t> head, upos, dw;
    head.alloc(nnz + 1);
    upos.alloc(nnz + 1);
    dw.alloc(W + 1);
    ACC_HIP(hipMemset(head.p + nnz, 0, sizeof(int32_t)));
    ACC_HIP(hipMemset(dw.p, 0, sizeof(int32_t) * (W + 1)));
    hipLaunchKernelGGL(mark_heads_kernel, dim3(blocks_for(nnz, 256)), dim3(256), 0, 0, nnz, sorted.p, head.p);
    exclusive_scan_i32(tmp, head.p, upos.p, nnz + 1);
    int32_t n_unique = 0;
    ACC_HIP(hipMemcpy(&n_unique, upos.p + nnz, sizeof(int32_t), hipMemcpyDeviceToHost));
    DevBuf<uint64_t> uniq;
    uniq.alloc(n_unique);
    hipLaunchKernelGGL(compact_heads_kernel, dim3(blocks_for(nnz, 256)), dim3(256), 0, 0, nnz, sorted.p, head.p,
                       upos.p, uniq.p);
    sorted.release();
    head.release();
    upos.release();

    DevBuf<int32_t> tw, ustart;
    tw.alloc(W + 1);
    ustart.alloc(W + 1);
    ACC_HIP(hipMemset(tw.p, 0, sizeof(int32_t) * (W + 1)));
    hipLaunchKernelGGL(window_starts_kernel, dim3(blocks_for(W + 1, 256)), dim3(256), 0, 0, W, (int64_t)n_unique, uniq.p,
                       colbits, ustart.p);
    hipLaunchKernelGGL(distinct_per_window_kernel, dim3(blocks_for(W, 256)), dim3(256), 0, 0, W, ustart.p, dw.p);
    hipLaunchKernelGGL(tiles_per_window_kernel, dim3(blocks_for(W, 256)), dim3(256), 0, 0, W, dw.p, TW, tw.p);
    exclusive_scan_i32(tmp, tw.p, out.row_window_offset.p, W + 1);
    int32_t T32 = 0;
    ACC_HIP(hipMemcpy(&T32, out.row_window_offset.p + W, sizeof(int32_t), hipMemcpyDeviceToHost));
    const int64_t T = T32;
    out.T = T;
    out.sum_dw = n_unique;
    if (tiles_only) return;
    if (T * TW >= ((int64_t)1 << 31)) fail(ACC_SPMM_ERR_UNSUPPORTED, "tile count exceeds 32-bit SparseAToB indexing");
    tw.release();
    dw.release();

    // 5. SparseAToB
    out.sparse_a_to_b.alloc(T * TW);
    hipLaunchKernelGGL(fill_a2b_kernel, dim3((unsigned)W), dim3(64), 0, 0, out.row_window_offset.p, ustart.p, uniq.p, TW,
                       (((uint64_t)1 << colbits) - 1), out.sparse_a_to_b.p);

    // 6. TCLocalBit
    out.tc_local_bit.alloc(T * NW);
    ACC_HIP(hipMemset(out.tc_local_bit.p, 0, sizeof(uint64_t) * T * NW));
    DevBuf<int32_t> tile_of;
    DevBuf<uint16_t> bit_of;
    tile_of.alloc(nnz);
    bit_of.alloc(nnz);
    hipLaunchKernelGGL(set_bits_kernel, dim3(blocks_for(M, 4)), dim3(256), 0, 0, M, d_rowptr, d_colidx, d_perm,
                       new_rowptr.p, out.row_window_offset.p, ustart.p, uniq.p, WH, TW, NW, colbits,
                       reinterpret_cast<unsigned long long*>(out.tc_local_bit.p), tile_of.p, bit_of.p);
    uniq.release();
    ustart.release();

    // 7. TCOffset
    DevBuf<int32_t> cnt;
    cnt.alloc(T + 1);
    ACC_HIP(hipMemset(cnt.p + T, 0, sizeof(int32_t)));
    out.tc_offset.alloc(T + 1);
    hipLaunchKernelGGL(tile_popcount_kernel, dim3(blocks_for(T, 256)), dim3(256), 0, 0, T, out.tc_local_bit.p, NW, cnt.p);
    exclusive_scan_i32(tmp, cnt.p, out.tc_offset.p, T + 1);
    cnt.release();

    // 8. values (8 halves of zero padding: the runtime kernel reads up to 4 past a tile's end)
    out.vals.alloc(nnz + 16);   // slack: the tile kernel's span loads read up to ten values past a lane's first
    ACC_HIP(hipMemset(out.vals.p + nnz, 0, 32));
    if (entry_of) entry_of->alloc(nnz);
    hipLaunchKernelGGL(scatter_values_kernel, dim3(blocks_for(M, 4)), dim3(256), 0, 0, M, d_rowptr, d_vals, d_perm,
                       new_rowptr.p, tile_of.p, bit_of.p, out.tc_local_bit.p, NW, out.tc_offset.p, out.vals.p,
                       entry_of ? entry_of->p : nullptr);
    ACC_HIP(hipGetLastError());
    ACC_HIP(hipDeviceSynchronize());
}

}  // namespace accspmm
