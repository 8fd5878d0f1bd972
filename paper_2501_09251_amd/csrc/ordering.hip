// Step II of the data-affinity reordering (paper Section 3.2, Algorithm 1: ordering
// generation) on the GPU.
//
// Input: the dendrogram's leaf sequence `seq` (M rows) cut into segments (seg_start).
// Inside a segment the next row of the chain is the unvisited row that shares the most
// column indices with the current row (at least one; ties: the earliest in the sequence);
// when no row shares a column the chain ends and the scan resumes at the first unvisited
// row.  Segments are independent, so one workgroup walks one segment.
//
// To count shared columns without intersecting row against row, an inverted index of the
// whole matrix is built once with device-wide primitives: every stored entry gets the key
// (segment, column); after a radix sort, entries with equal keys are adjacent ("runs"), and
// every entry remembers its run.  A chain step then walks, for each entry of the current
// row, that entry's run, and bumps a counter in LDS for every unvisited row in it.
#include "device_util.h"

namespace accspmm {
namespace {

using namespace detail;

constexpr int kChainThreads = 256;

__global__ void seq_row_lengths_kernel(int64_t M, const int32_t* __restrict__ rowptr, const int32_t* __restrict__ seq,
                                       int32_t* __restrict__ len) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < M) {
        int32_t i = seq[p];
        len[p] = rowptr[i + 1] - rowptr[i];
    }
}

// segment of every sequence position: seg_of[p] = s with seg_start[s] <= p < seg_start[s+1]
__global__ void segment_of_kernel(int64_t M, int64_t nseg, const int32_t* __restrict__ seg_start,
                                  int32_t* __restrict__ seg_of) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= M) return;
    int64_t lo = 0, hi = nseg;  // last s with seg_start[s] <= p
    while (hi - lo > 1) {
        int64_t mid = (lo + hi) >> 1;
        if (seg_start[mid] <= p) lo = mid; else hi = mid;
    }
    seg_of[p] = (int32_t)lo;
}

// one wavefront per sequence position: key (segment, column) and local position of each entry
__global__ __launch_bounds__(256) void make_entry_keys_kernel(int64_t M, const int32_t* __restrict__ rowptr,
                                                              const int32_t* __restrict__ colidx,
                                                              const int32_t* __restrict__ seq,
                                                              const int32_t* __restrict__ seq_rowptr,
                                                              const int32_t* __restrict__ seg_of,
                                                              const int32_t* __restrict__ seg_start, int32_t colbits,
                                                              uint64_t* __restrict__ keys, uint32_t* __restrict__ entry_id,
                                                              uint16_t* __restrict__ entry_q) {
    int64_t p = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (p >= M) return;
    const int lane = threadIdx.x & 63;
    const int32_t s = seg_of[p];
    const uint16_t q = (uint16_t)(p - seg_start[s]);
    const int32_t src = rowptr[seq[p]], dst = seq_rowptr[p], len = seq_rowptr[p + 1] - dst;
    const uint64_t hi = (uint64_t)s << colbits;
    for (int32_t k = lane; k < len; k += 64) {
        keys[dst + k] = hi | (uint32_t)colidx[src + k];
        entry_id[dst + k] = (uint32_t)(dst + k);
        entry_q[dst + k] = q;
    }
}

// run_id[i] = (inclusive count of heads up to i) - 1.  For every sorted position: remember
// the run's first position, the run of the originating entry, and the entry's local row.
__global__ void scatter_runs_kernel(int64_t n, const int32_t* __restrict__ head, const int32_t* __restrict__ head_excl,
                                    const uint32_t* __restrict__ sorted_entry, const uint16_t* __restrict__ entry_q,
                                    int32_t* __restrict__ run_begin, int32_t* __restrict__ entry_run,
                                    uint16_t* __restrict__ sorted_q) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t run = head_excl[i] + head[i] - 1;
    if (head[i]) run_begin[run] = (int32_t)i;
    const uint32_t e = sorted_entry[i];
    entry_run[e] = run;
    sorted_q[i] = entry_q[e];
}

__global__ void singleton_segments_kernel(int64_t nseg, const int32_t* __restrict__ seg_start,
                                          const int32_t* __restrict__ seq, int32_t* __restrict__ perm) {
    int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s < nseg && seg_start[s + 1] - seg_start[s] == 1) perm[seg_start[s]] = seq[seg_start[s]];
}

// One workgroup per multi-row segment.  MAXN = capacity of the LDS arrays (>= segment length).
template <int MAXN>
__global__ __launch_bounds__(kChainThreads) void chain_segments_kernel(
    const int32_t* __restrict__ multi_segments, const int32_t* __restrict__ seg_start, const int32_t* __restrict__ seq,
    const int32_t* __restrict__ seq_rowptr, const int32_t* __restrict__ entry_run, const int32_t* __restrict__ run_begin,
    const uint16_t* __restrict__ sorted_q, int32_t* __restrict__ perm) {
    __shared__ uint32_t count[MAXN];
    __shared__ uint8_t visited[MAXN];
    __shared__ uint32_t wave_best[kChainThreads / 64];
    __shared__ int32_t s_next;  // next chain head, or -1
    const int s = multi_segments[blockIdx.x];
    const int b = seg_start[s], n = seg_start[s + 1] - b;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int q = tid; q < n; q += kChainThreads) { count[q] = 0; visited[q] = 0; }
    __syncthreads();
    int out = b;   // next new id (same value in every thread)
    int cur = 0;   // scan position for the first unvisited row (same value in every thread)
    while (cur < n) {
        if (visited[cur]) { ++cur; continue; }
        int v = cur;
        for (;;) {  // one chain
            __syncthreads();  // counts are zero, previous step's reads of `visited` are done
            if (tid == 0) { visited[v] = 1; perm[out] = seq[b + v]; }
            ++out;
            __syncthreads();
            // every entry of row v: walk its run (the rows of this segment holding that column)
            const int e0 = seq_rowptr[b + v], e1 = seq_rowptr[b + v + 1];
            for (int e = e0 + wave; e < e1; e += kChainThreads / 64) {
                const int run = entry_run[e];
                const int r0 = run_begin[run], r1 = run_begin[run + 1];
                for (int i = r0 + lane; i < r1; i += 64) {
                    const int q = sorted_q[i];
                    if (!visited[q]) atomicAdd(&count[q], 1u);
                }
            }
            __syncthreads();
            // arg max of (count, earliest position); clears the counters on the way
            uint32_t best = 0;
            for (int q = tid; q < n; q += kChainThreads) {
                const uint32_t c = count[q];
                if (c) {
                    count[q] = 0;
                    const uint32_t key = (c << 12) | (uint32_t)(MAXN - 1 - q);  // c <= 2^20 - 1 checked on the host
                    best = key > best ? key : best;
                }
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const uint32_t o = __shfl_xor(best, off, 64);
                best = o > best ? o : best;
            }
            if (lane == 0) wave_best[wave] = best;
            __syncthreads();
            if (tid == 0) {
                uint32_t bb = 0;
                for (int k = 0; k < kChainThreads / 64; ++k) bb = wave_best[k] > bb ? wave_best[k] : bb;
                s_next = bb ? (MAXN - 1 - (int)(bb & 0xFFFu)) : -1;
            }
            __syncthreads();
            const int nxt = s_next;
            if (nxt < 0) break;
            v = nxt;
        }
        ++cur;
    }
}

}  // namespace

void ordering_on_device(int64_t M, int64_t K, int64_t nnz, const int32_t* d_rowptr, const int32_t* d_colidx,
                        const std::vector<int32_t>& seq, const std::vector<int64_t>& seg_start, int32_t seg_len,
                        int32_t max_row_len, DevBuf<int32_t>& d_perm) {
    static_assert(kChainThreads % 64 == 0, "whole wavefronts");
    constexpr int kMaxSegLen = 4096;
    if (seg_len > kMaxSegLen) fail(ACC_SPMM_ERR_UNSUPPORTED, "segment_length above 4096 is not supported");
    // the arg-max key packs (count << 12 | position): counts are bounded by the longest row
    if ((int64_t)max_row_len >= ((int64_t)1 << 20)) fail(ACC_SPMM_ERR_UNSUPPORTED, "a row with 2^20 or more entries cannot be reordered");
    const int64_t nseg = (int64_t)seg_start.size() - 1;
    const int colbits = bits_for(K), segbits = bits_for(nseg);
    if (colbits + segbits > 64) fail(ACC_SPMM_ERR_UNSUPPORTED, "matrix too large for the reordering keys");
    d_perm.alloc(M);
    if (M == 0) return;

    std::vector<int32_t> seg32(seg_start.begin(), seg_start.end());
    std::vector<int32_t> multi;
    for (int64_t s = 0; s < nseg; ++s)
        if (seg_start[s + 1] - seg_start[s] > 1) multi.push_back((int32_t)s);
    DevBuf<int32_t> d_seq, d_seg, d_multi;
    d_seq.upload(seq.data(), M);
    d_seg.upload(seg32.data(), seg32.size());
    d_multi.upload(multi.data(), multi.size());
    hipLaunchKernelGGL(singleton_segments_kernel, dim3(blocks_for(nseg, 256)), dim3(256), 0, 0, nseg, d_seg.p, d_seq.p, d_perm.p);
    if (multi.empty()) {
        ACC_HIP(hipDeviceSynchronize());
        return;
    }
    Scratch tmp;
    auto scan = [&](const int32_t* in, int32_t* out, size_t n) { exclusive_scan_i32(tmp, in, out, n); };

    // entry ranges of the rows in sequence order
    DevBuf<int32_t> len, seq_rowptr, seg_of;
    len.alloc(M + 1);
    seq_rowptr.alloc(M + 1);
    seg_of.alloc(M);
    ACC_HIP(hipMemset(len.p + M, 0, sizeof(int32_t)));
    hipLaunchKernelGGL(seq_row_lengths_kernel, dim3(blocks_for(M, 256)), dim3(256), 0, 0, M, d_rowptr, d_seq.p, len.p);
    scan(len.p, seq_rowptr.p, M + 1);
    len.release();
    hipLaunchKernelGGL(segment_of_kernel, dim3(blocks_for(M, 256)), dim3(256), 0, 0, M, nseg, d_seg.p, seg_of.p);

    // inverted index: sort the entries by (segment, column)
    DevBuf<uint64_t> keys, sorted_keys;
    DevBuf<uint32_t> entry_id, sorted_entry;
    DevBuf<uint16_t> entry_q, sorted_q;
    keys.alloc(nnz);
    sorted_keys.alloc(nnz);
    entry_id.alloc(nnz);
    sorted_entry.alloc(nnz);
    entry_q.alloc(nnz);
    hipLaunchKernelGGL(make_entry_keys_kernel, dim3(blocks_for(M, 4)), dim3(256), 0, 0, M, d_rowptr, d_colidx, d_seq.p,
                       seq_rowptr.p, seg_of.p, d_seg.p, colbits, keys.p, entry_id.p, entry_q.p);
    {
        size_t bytes = 0;
        ACC_HIP(rocprim::radix_sort_pairs(nullptr, bytes, keys.p, sorted_keys.p, entry_id.p, sorted_entry.p, (size_t)nnz, 0u,
                                          (unsigned)(colbits + segbits)));
        ACC_HIP(rocprim::radix_sort_pairs(tmp.get(bytes), bytes, keys.p, sorted_keys.p, entry_id.p, sorted_entry.p,
                                          (size_t)nnz, 0u, (unsigned)(colbits + segbits)));
    }
    keys.release();
    entry_id.release();
    seg_of.release();

    DevBuf<int32_t> head, head_excl, run_begin, entry_run;
    head.alloc(nnz + 1);
    head_excl.alloc(nnz + 1);
    ACC_HIP(hipMemset(head.p + nnz, 0, sizeof(int32_t)));
    hipLaunchKernelGGL(mark_heads_kernel, dim3(blocks_for(nnz, 256)), dim3(256), 0, 0, nnz, sorted_keys.p, head.p);
    scan(head.p, head_excl.p, nnz + 1);
    sorted_keys.release();
    int32_t n_runs = 0;
    ACC_HIP(hipMemcpy(&n_runs, head_excl.p + nnz, sizeof(int32_t), hipMemcpyDeviceToHost));
    run_begin.alloc((size_t)n_runs + 1);
    const int32_t nnz32 = (int32_t)nnz;
    ACC_HIP(hipMemcpy(run_begin.p + n_runs, &nnz32, sizeof(int32_t), hipMemcpyHostToDevice));
    entry_run.alloc(nnz);
    sorted_q.alloc(nnz);
    hipLaunchKernelGGL(scatter_runs_kernel, dim3(blocks_for(nnz, 256)), dim3(256), 0, 0, nnz, head.p, head_excl.p,
                       sorted_entry.p, entry_q.p, run_begin.p, entry_run.p, sorted_q.p);
    head.release();
    head_excl.release();
    sorted_entry.release();
    entry_q.release();

    const dim3 grid((unsigned)multi.size()), block(kChainThreads);
    if (seg_len <= 1024)
        hipLaunchKernelGGL(chain_segments_kernel<1024>, grid, block, 0, 0, d_multi.p, d_seg.p, d_seq.p, seq_rowptr.p,
                           entry_run.p, run_begin.p, sorted_q.p, d_perm.p);
    else
        hipLaunchKernelGGL(chain_segments_kernel<kMaxSegLen>, grid, block, 0, 0, d_multi.p, d_seg.p, d_seq.p, seq_rowptr.p,
                           entry_run.p, run_begin.p, sorted_q.p, d_perm.p);
    ACC_HIP(hipGetLastError());
    ACC_HIP(hipDeviceSynchronize());
}

}  // namespace accspmm
