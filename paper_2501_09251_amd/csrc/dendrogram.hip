// Step I of the data-affinity reordering (paper Section 3.2, Algorithm 1: dendrogram
// construction) on the GPU, with exactly the result of the sequential definition.
//
// The definition is sequential: vertices are visited in ascending degree (ties by id) and a
// vertex's decision (which neighbouring community maximises the gain s = w*2m - d_u*d_v of Eq. 1,
// read as the modularity gain; merge iff s > 0; ties to the lower community id) depends on every
// earlier merge.  It is reproduced in rounds.  A round takes the next P vertices of the order
// ("slots"), decides each of them against the state as it was when the round began, and then
// keeps the longest prefix of slots whose decision the earlier slots of the same round cannot
// have changed.  Slot i stands iff
//   (a) none of its candidate communities is the vertex of an earlier slot that merges
//       (that community's root would have changed),
//   (b) no earlier slot merges into its own vertex (its edge list and degree would have changed),
//   (c) its chosen community b received no degree from earlier slots, or it still wins after it
//       did: merges only raise the degree sums of their targets, which only lowers scores, so a
//       winner whose own score is untouched stays the winner, and one whose score dropped to
//       s' stays the winner if s' > 0 and s' beats the runner-up's score of the round's start.
// The first slot of a round always stands, so every round advances.  Everything before the first
// slot that fails is committed (its decision equals the sequential one by induction), the rest is
// decided again in the next round.  (c) may fail a slot whose decision would in fact have stood;
// that costs a round, never the result.
//
// A community's edge list, as of its vertex's turn, is its own adjacency plus the lists of the
// vertices merged into it (each a list of (community, weight) pairs as of that vertex's turn);
// endpoints are mapped to their present roots when the list is read.  The lists of the vertices
// that one round merges into one target are stored as one chunk; a target's chunks are found
// through a chain of small directory blocks.
#include "device_util.h"

namespace accspmm {
namespace {

using namespace detail;

constexpr int kSlots = 2048;          // most vertices decided per round
constexpr int kRowWords = kSlots / 32;
constexpr int kSmallRecords = 512;    // a slot with at most this many edge records is decided by one wavefront
constexpr int kHashSize = 1024;       // entries of that wavefront's hash table in LDS
constexpr int kUnit = 4096;           // edge records per thread block for larger slots
constexpr int kLargeBlocks = 1024;    // grid of the kernels that walk those units
constexpr int kMaxDense = 64;         // larger slots per round (each owns a weight array over all vertices)
constexpr int kDescPerBlock = 8;      // chunk descriptors per directory block
constexpr long long kAdjacencyFlag = 1ll << 62;

constexpr int kClassNone = 0, kClassSmall = 1, kClassLarge = 2, kClassSkipped = 3;

struct Rec {
    int32_t to;
    uint32_t w;
};

struct Ctl {                 // round control, lives in device memory
    long long pos;           // vertices of the order that have had their turn
    long long work;          // edge records read by those turns, +1 per turn
    long long work_at_last;  // the same count when the last vertex of the order began its turn
    long long arena_used;
    long long rounds;
    int P;                   // slots of the next round
    int n_prepared, n_eval;  // slots of this round; those among them that got the memory they need
    int n_units;
    int last_cut;            // slots the last commit kept
    int blk_used;
    int overflow;            // a memory pool was exhausted: nothing more is committed
    int pad;
};

struct DS {
    long long M, two_m;
    const long long* gptr;
    const int32_t* gadj;
    const int32_t* order;
    const int32_t* idx;
    int32_t* parent;
    int32_t* up;
    long long* dsum;
    int32_t* head;
    int32_t* blk_next;
    int32_t* blk_count;
    long long* blk_off;
    int32_t* blk_len;
    int32_t blk_cap;
    Rec* arena;
    long long arena_cap;
    Ctl* ctl;
    int32_t* slot_of;
    int32_t *s_v, *s_nrec, *s_class, *s_dense, *s_desc_off, *s_ndesc, *s_unit0, *s_nunits, *s_nt, *s_best, *s_store;
    long long *s_cand_off, *s_score, *s_second, *s_dv, *s_chunk_off;
    uint32_t* bits;
    int32_t* row_dirty;
    Rec* scand;
    Rec* cand;
    long long cand_cap;
    long long* d_off;
    int32_t* d_len;
    long long* d_start;
    int32_t desc_cap;
    int32_t* unit_slot;
    int32_t unit_cap;
    int32_t* u_best;
    long long *u_score, *u_second;
    uint32_t* dense;
    int32_t n_dense;
};

// Root of x's community.  Links only ever point from a vertex that has had its turn to what was a
// root then, so the walk ends; the hop limit is a guard that turns a broken link structure into a
// wrong answer (which the caller's consistency check reports) instead of an endless loop.
constexpr int kMaxHops = 1 << 22;
__device__ __forceinline__ int32_t find_root(const int32_t* up, int32_t x) {
    int32_t p = up[x];
    for (int hop = 0; p != x && hop < kMaxHops; ++hop) {
        x = p;
        p = up[x];
    }
    return x;
}

// (score, community) pairs: the better one has the larger score, ties go to the lower id
struct Best {
    long long s, second;   // best score; best score among the other candidates (LLONG_MIN if none)
    int32_t r;             // -1: no candidate
};
constexpr long long kNoScore = (long long)0x8000000000000000ull;

__device__ __forceinline__ void best_add(Best& b, long long s, int32_t r) {
    if (b.r < 0 || s > b.s || (s == b.s && r < b.r)) {
        if (b.r >= 0 && b.s > b.second) b.second = b.s;
        b.s = s;
        b.r = r;
    } else if (s > b.second) {
        b.second = s;
    }
}
__device__ __forceinline__ void best_join(Best& a, const Best& o) {
    if (o.r < 0) return;
    if (o.second > a.second) a.second = o.second;
    best_add(a, o.s, o.r);
}
__device__ __forceinline__ Best best_wave_reduce(Best b) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        Best x;
        x.s = __shfl_xor(b.s, o);
        x.second = __shfl_xor(b.second, o);
        x.r = __shfl_xor(b.r, o);
        best_join(b, x);
    }
    return b;
}

__global__ void init_state_kernel(long long M, const long long* __restrict__ gptr, const int32_t* __restrict__ order,
                                  int32_t* idx, int32_t* parent, int32_t* up, long long* dsum, int32_t* head,
                                  int32_t* slot_of) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M) return;
    idx[order[i]] = (int32_t)i;
    parent[i] = -1;
    up[i] = (int32_t)i;
    dsum[i] = gptr[i + 1] - gptr[i];
    head[i] = -1;
    slot_of[i] = -1;
}

__global__ void degree_keys_kernel(long long M, const long long* __restrict__ gptr, uint32_t* key, int32_t* id) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M) return;
    key[i] = (uint32_t)(gptr[i + 1] - gptr[i]);
    id[i] = (int32_t)i;
}

// Shortens the paths that find_root walks; any mix of old and new links leads to the same roots.
__global__ void compress_paths_kernel(long long M, int32_t* up) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < M) up[i] = find_root(up, (int32_t)i);
}

// exclusive prefix sum over the block's 1024 threads; `total` gets the sum
__device__ __forceinline__ long long block_scan_1024(long long x, long long* sh, long long& total) {
    const int t = threadIdx.x;
    sh[t] = x;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
        const long long y = t >= o ? sh[t - o] : 0;
        __syncthreads();
        sh[t] += y;
        __syncthreads();
    }
    const long long incl = sh[t];
    total = sh[1023];
    __syncthreads();
    return incl - x;
}

// Round step 1 (one block of 1024 threads, two consecutive slots per thread): the round's vertices,
// the size of their edge lists, and, in slot order, the memory the larger slots need.
__global__ __launch_bounds__(1024) void prepare_round_kernel(DS d) {
    __shared__ long long sh[1024];
    __shared__ int first_unfit;
    const int t = threadIdx.x;
    Ctl* const ctl = d.ctl;
    const long long pos = ctl->pos;
    const int P = ctl->P;
    const int n = (int)(d.M - pos < (long long)P ? d.M - pos : (long long)P);
    if (t == 0) first_unfit = n;
    int v[2], nrec[2], ndesc[2], cls[2];
    for (int k = 0; k < 2; ++k) {
        const int i = 2 * t + k;
        v[k] = -1; nrec[k] = 0; ndesc[k] = 0; cls[k] = kClassNone;
        if (i >= n) continue;
        const int32_t x = d.order[pos + i];
        v[k] = x;
        d.slot_of[x] = i;
        d.s_v[i] = x;
        const long long deg = d.gptr[x + 1] - d.gptr[x];
        long long records = deg;
        int descs = deg > 0 ? 1 : 0;
        int guard = 0;
        for (int32_t b = d.head[x]; b >= 0 && guard <= d.blk_cap; b = d.blk_next[b], ++guard) {
            const int c = d.blk_count[b];
            for (int e = 0; e < c; ++e) records += d.blk_len[(long long)b * kDescPerBlock + e];
            descs += c;
        }
        nrec[k] = (int)records;
        ndesc[k] = descs;
        cls[k] = records <= kSmallRecords ? kClassSmall : kClassLarge;
    }
    // what the larger slots need, as exclusive prefix sums in slot order
    auto need = [&](int k, int what) -> long long {
        if (cls[k] != kClassLarge) return 0;
        switch (what) {
            case 0: return 1;
            case 1: return nrec[k];
            case 2: return ndesc[k];
            default: return (nrec[k] + kUnit - 1) / kUnit;
        }
    };
    long long pre[4][2], tot[4];
    for (int what = 0; what < 4; ++what) {
        const long long a = need(0, what), b = need(1, what);
        const long long ex = block_scan_1024(a + b, sh, tot[what]);
        pre[what][0] = ex;
        pre[what][1] = ex + a;
    }
    const long long cap[4] = {(long long)d.n_dense, d.cand_cap, (long long)d.desc_cap, (long long)d.unit_cap};
    for (int k = 0; k < 2; ++k) {
        const int i = 2 * t + k;
        if (i >= n) continue;
        bool fit = true;
        for (int what = 0; what < 4; ++what) fit = fit && pre[what][k] + need(k, what) <= cap[what];
        if (!fit) atomicMin(&first_unfit, i);
    }
    __syncthreads();
    const int n_eval = first_unfit;
    long long units_total = 0;
    for (int k = 0; k < 2; ++k) {
        const int i = 2 * t + k;
        if (i >= n) continue;
        if (i >= n_eval) cls[k] = kClassSkipped;
        d.s_class[i] = cls[k];
        d.s_nrec[i] = nrec[k];
        d.s_nt[i] = 0;
        d.s_store[i] = 0;
        if (cls[k] != kClassLarge) continue;
        const int32_t x = v[k];
        const int nunits = (nrec[k] + kUnit - 1) / kUnit;
        d.s_dense[i] = (int)pre[0][k];
        d.s_cand_off[i] = pre[1][k];
        d.s_desc_off[i] = (int)pre[2][k];
        d.s_ndesc[i] = ndesc[k];
        d.s_unit0[i] = (int)pre[3][k];
        d.s_nunits[i] = nunits;
        units_total += nunits;
        for (int u = 0; u < nunits; ++u) d.unit_slot[pre[3][k] + u] = i;
        // descriptors: the vertex's own adjacency first, then its chunks
        long long j = pre[2][k], start = 0;
        const long long deg = d.gptr[x + 1] - d.gptr[x];
        if (deg > 0) {
            d.d_off[j] = d.gptr[x] | kAdjacencyFlag;
            d.d_len[j] = (int)deg;
            d.d_start[j] = 0;
            start = deg;
            ++j;
        }
        int guard = 0;
        for (int32_t b = d.head[x]; b >= 0 && guard <= d.blk_cap; b = d.blk_next[b], ++guard) {
            const int c = d.blk_count[b];
            for (int e = 0; e < c; ++e) {
                d.d_off[j] = d.blk_off[(long long)b * kDescPerBlock + e];
                d.d_len[j] = d.blk_len[(long long)b * kDescPerBlock + e];
                d.d_start[j] = start;
                start += d.d_len[j];
                ++j;
            }
        }
    }
    long long all_units;
    (void)block_scan_1024(units_total, sh, all_units);
    if (t == 0) {
        ctl->n_prepared = n;
        ctl->n_eval = n_eval;
        ctl->n_units = (int)all_units;
    }
}

// Round step 2a: one wavefront (a block of 64 threads) decides one small slot.  The weights towards
// the neighbouring communities are summed in a hash table in LDS.
__global__ __launch_bounds__(64) void decide_small_kernel(DS d) {
    __shared__ int32_t hkey[kHashSize];
    __shared__ uint32_t hval[kHashSize];
    const int i = blockIdx.x, lane = threadIdx.x;
    if (i >= d.ctl->n_eval || d.s_class[i] != kClassSmall) return;
    const int32_t v = d.s_v[i];
    for (int e = lane; e < kHashSize; e += 64) { hkey[e] = -1; hval[e] = 0; }
    __syncthreads();
    auto add = [&](int32_t to, uint32_t w) {
        const int32_t r = find_root(d.up, to);
        if (r == v) return;
        uint32_t h = ((uint32_t)r * 2654435761u) >> 22;   // 10 bits
        for (int probe = 0; probe < kHashSize; ++probe) {
            const int32_t k = atomicCAS(&hkey[h], -1, r);
            if (k == -1 || k == r) { atomicAdd(&hval[h], w); return; }
            h = (h + 1) & (kHashSize - 1);
        }
    };
    const long long gb = d.gptr[v], ge = d.gptr[v + 1];
    for (long long p = gb + lane; p < ge; p += 64) add(d.gadj[p], 1u);
    int guard = 0;
    for (int32_t b = d.head[v]; b >= 0 && guard <= d.blk_cap; b = d.blk_next[b], ++guard) {
        const int c = d.blk_count[b];
        for (int e = 0; e < c; ++e) {
            const Rec* list = d.arena + d.blk_off[(long long)b * kDescPerBlock + e];
            const int len = d.blk_len[(long long)b * kDescPerBlock + e];
            for (int q = lane; q < len; q += 64) add(list[q].to, list[q].w);
        }
    }
    __syncthreads();
    const long long dv = d.dsum[v];
    Best best{kNoScore, kNoScore, -1};
    int count = 0;
    bool dirty = false;
    Rec* const out = d.scand + (long long)i * kSmallRecords;
    for (int e0 = 0; e0 < kHashSize; e0 += 64) {
        const int32_t r = hkey[e0 + lane];
        const bool have = r >= 0;
        const uint32_t w = hval[e0 + lane];
        if (have) {
            best_add(best, (long long)w * d.two_m - d.dsum[r] * dv, r);
            const int j = d.slot_of[r];
            if (j >= 0) { atomicOr(&d.bits[(long long)i * kRowWords + (j >> 5)], 1u << (j & 31)); dirty = true; }
        }
        const unsigned long long m = __ballot(have);
        if (have) out[count + __popcll(m & ((1ull << lane) - 1ull))] = Rec{r, w};
        count += __popcll(m);
    }
    best = best_wave_reduce(best);
    if (__ballot(dirty) && lane == 0) d.row_dirty[i] = 1;
    if (lane == 0) {
        d.s_nt[i] = count;
        d.s_best[i] = best.r;
        d.s_score[i] = best.s;
        d.s_second[i] = best.second;
        d.s_dv[i] = dv;
    }
}

// Round step 2b: the edge records of the larger slots, kUnit per block, summed into the slot's
// weight array over all vertices; the communities met for the first time are appended to the
// slot's candidate list.
__global__ __launch_bounds__(256) void accumulate_large_kernel(DS d) {
    const int n_units = d.ctl->n_units;
    for (int u = blockIdx.x; u < n_units; u += gridDim.x) {
        const int i = d.unit_slot[u];
        const int k = u - d.s_unit0[i];
        const int32_t v = d.s_v[i];
        const int nrec = d.s_nrec[i];
        const long long dbase = d.s_desc_off[i];
        const int nd = d.s_ndesc[i];
        uint32_t* const weight = d.dense + (long long)d.s_dense[i] * d.M;
        Rec* const cand = d.cand + d.s_cand_off[i];
        const int p_end = (k + 1) * kUnit < nrec ? (k + 1) * kUnit : nrec;
        for (int p = k * kUnit + (int)threadIdx.x; p < p_end; p += 256) {
            int lo = 0, hi = nd - 1;          // last descriptor that starts at or before p
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (d.d_start[dbase + mid] <= p) lo = mid; else hi = mid - 1;
            }
            const long long q = p - d.d_start[dbase + lo];
            const long long off = d.d_off[dbase + lo];
            int32_t to;
            uint32_t w;
            if (off & kAdjacencyFlag) { to = d.gadj[(off & ~kAdjacencyFlag) + q]; w = 1u; }
            else { const Rec r = d.arena[off + q]; to = r.to; w = r.w; }
            const int32_t r = find_root(d.up, to);
            if (r == v) continue;
            if (atomicAdd(&weight[r], w) == 0u) cand[atomicAdd(&d.s_nt[i], 1)].to = r;
        }
    }
}

// Round step 2c: scores of the larger slots' candidates (kUnit per block), the block's best and
// runner-up; the weight array is cleared on the way.
__global__ __launch_bounds__(256) void score_large_kernel(DS d) {
    __shared__ long long sh_s[4], sh_second[4];
    __shared__ int32_t sh_r[4];
    const int n_units = d.ctl->n_units;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int u = blockIdx.x; u < n_units; u += gridDim.x) {
        const int i = d.unit_slot[u];
        const int k = u - d.s_unit0[i];
        const int32_t v = d.s_v[i];
        const int nt = d.s_nt[i];
        const long long dv = d.dsum[v];
        uint32_t* const weight = d.dense + (long long)d.s_dense[i] * d.M;
        Rec* const cand = d.cand + d.s_cand_off[i];
        const int j_end = (k + 1) * kUnit < nt ? (k + 1) * kUnit : nt;
        Best best{kNoScore, kNoScore, -1};
        bool dirty = false;
        for (int j = k * kUnit + (int)threadIdx.x; j < j_end; j += 256) {
            const int32_t r = cand[j].to;
            const uint32_t w = weight[r];
            cand[j].w = w;
            weight[r] = 0u;
            best_add(best, (long long)w * d.two_m - d.dsum[r] * dv, r);
            const int sj = d.slot_of[r];
            if (sj >= 0) { atomicOr(&d.bits[(long long)i * kRowWords + (sj >> 5)], 1u << (sj & 31)); dirty = true; }
        }
        if (dirty) d.row_dirty[i] = 1;
        best = best_wave_reduce(best);
        if (lane == 0) { sh_s[wave] = best.s; sh_second[wave] = best.second; sh_r[wave] = best.r; }
        __syncthreads();
        if (threadIdx.x == 0) {
            Best all{sh_s[0], sh_second[0], sh_r[0]};
            for (int w2 = 1; w2 < 4; ++w2) best_join(all, Best{sh_s[w2], sh_second[w2], sh_r[w2]});
            d.u_best[u] = all.r;
            d.u_score[u] = all.s;
            d.u_second[u] = all.second;
        }
        __syncthreads();
    }
}

// ascending bitonic sort of 2048 keys in LDS by 1024 threads
__device__ __forceinline__ void bitonic_sort_2048(unsigned long long* key) {
    const int t = threadIdx.x;
    for (int size = 2; size <= kSlots; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            const int lo = ((t & ~(stride - 1)) << 1) | (t & (stride - 1));
            const int hi = lo + stride;
            const bool up = (lo & size) == 0;
            const unsigned long long a = key[lo], b = key[hi];
            if ((a > b) == up) { key[lo] = b; key[hi] = a; }
        }
    }
    __syncthreads();
}

// inclusive sums of val inside runs (a run starts where head is set); 2048 positions, two per thread
__device__ __forceinline__ void segmented_scan_2048(long long* val, uint8_t* flag, const uint8_t* head) {
    const int t = threadIdx.x;
    for (int k = 0; k < 2; ++k) flag[t + k * 1024] = head[t + k * 1024];
    __syncthreads();
    for (int o = 1; o < kSlots; o <<= 1) {
        long long add[2];
        uint8_t f[2];
        for (int k = 0; k < 2; ++k) {
            const int p = t + k * 1024;
            add[k] = 0;
            f[k] = flag[p];
            if (p >= o && !flag[p]) { add[k] = val[p - o]; f[k] = flag[p - o]; }
        }
        __syncthreads();
        for (int k = 0; k < 2; ++k) {
            const int p = t + k * 1024;
            val[p] += add[k];
            flag[p] = f[k];
        }
        __syncthreads();
    }
}

// Round step 3 (one block of 1024 threads): which slots stand, and the commit of those.
__global__ __launch_bounds__(1024) void commit_round_kernel(DS d) {
    __shared__ unsigned long long key[kSlots];
    __shared__ long long val[kSlots];
    __shared__ long long aux[kSlots];            // reductions (first 1024 entries), then the runs' arena offsets
    __shared__ uint32_t mmask[kRowWords];
    __shared__ uint8_t inv[kSlots], head[kSlots], flag[kSlots];
    __shared__ int16_t pos_of_slot[kSlots], hpos[kSlots];   // sorted position of a slot; first position of a position's run
    __shared__ int cut_sh, overflow_sh;
    long long* const red = aux;
    long long* const run_base = aux;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    Ctl* const ctl = d.ctl;
    const int n_prepared = ctl->n_prepared, n_eval = ctl->n_eval;
    if (n_prepared == 0) return;
    if (t < kRowWords) mmask[t] = 0;
    if (t == 0) { cut_sh = n_eval; overflow_sh = 0; }
    __syncthreads();
    // results of the larger slots from their blocks' partial results; who merges
    for (int k = 0; k < 2; ++k) {
        const int i = t + k * 1024;
        inv[i] = 0;
        key[i] = ~0ull;
        if (i >= n_eval) continue;
        if (d.s_class[i] == kClassLarge) {
            Best all{kNoScore, kNoScore, -1};
            const int u0 = d.s_unit0[i], nu = d.s_nunits[i];
            for (int u = u0; u < u0 + nu; ++u) best_join(all, Best{d.u_score[u], d.u_second[u], d.u_best[u]});
            d.s_best[i] = all.r;
            d.s_score[i] = all.s;
            d.s_second[i] = all.second;
            d.s_dv[i] = d.dsum[d.s_v[i]];
        }
        if (d.s_best[i] >= 0 && d.s_score[i] > 0) {
            atomicOr(&mmask[i >> 5], 1u << (i & 31));
            key[i] = ((unsigned long long)(uint32_t)d.s_best[i] << 11) | (unsigned long long)i;
        }
    }
    __syncthreads();
    // (b) an earlier slot merges into this slot's vertex
    for (int k = 0; k < 2; ++k) {
        const int j = t + k * 1024;
        if (j >= n_eval || key[j] == ~0ull) continue;
        const int s = d.slot_of[d.s_best[j]];
        if (s > j && s < n_eval) inv[s] = 1;
    }
    // (a) a candidate community is the vertex of an earlier slot that merges
    for (int i = wave; i < n_eval; i += 16) {
        if (!d.row_dirty[i]) continue;
        const uint32_t word = d.bits[(long long)i * kRowWords + lane];
        const uint32_t below = lane < (i >> 5) ? 0xffffffffu : (lane == (i >> 5) ? ((1u << (i & 31)) - 1u) : 0u);
        if (__ballot((word & mmask[lane] & below) != 0u) && lane == 0) inv[i] = 1;
        d.bits[(long long)i * kRowWords + lane] = 0u;
        if (lane == 0) d.row_dirty[i] = 0;
    }
    // (c) degree that earlier slots add to the chosen community: merging slots sorted by (target, slot)
    bitonic_sort_2048(key);
    for (int k = 0; k < 2; ++k) {
        const int p = t + k * 1024;
        const unsigned long long kk = key[p];
        head[p] = p == 0 || (kk >> 11) != (key[p - 1] >> 11);
        val[p] = kk == ~0ull ? 0 : d.s_dv[(int)(kk & (kSlots - 1))];
        if (kk != ~0ull) pos_of_slot[(int)(kk & (kSlots - 1))] = (int16_t)p;
    }
    __syncthreads();
    // first position of every position's run: running maximum of the head positions
    for (int k = 0; k < 2; ++k) { const int p = t + k * 1024; hpos[p] = head[p] ? (int16_t)p : (int16_t)0; }
    __syncthreads();
    for (int o = 1; o < kSlots; o <<= 1) {
        int16_t m[2];
        for (int k = 0; k < 2; ++k) { const int p = t + k * 1024; m[k] = p >= o && hpos[p - o] > hpos[p] ? hpos[p - o] : hpos[p]; }
        __syncthreads();
        for (int k = 0; k < 2; ++k) hpos[t + k * 1024] = m[k];
        __syncthreads();
    }
    segmented_scan_2048(val, flag, head);
    for (int k = 0; k < 2; ++k) {
        const int p = t + k * 1024;
        const unsigned long long kk = key[p];
        if (kk == ~0ull) continue;
        const int i = (int)(kk & (kSlots - 1));
        const long long dv = d.s_dv[i];
        const long long before = val[p] - dv;      // degree added to the target by earlier slots
        if (before > 0) {
            const long long adjusted = d.s_score[i] - before * dv;
            if (!(adjusted > 0 && adjusted > d.s_second[i])) inv[i] = 1;
        }
    }
    __syncthreads();
    for (int k = 0; k < 2; ++k) {
        const int i = t + k * 1024;
        if (i < n_eval && inv[i]) atomicMin(&cut_sh, i);
    }
    __syncthreads();
    int cut = cut_sh;
    // edge lists to keep: those of committed merges whose target has its turn still ahead
    __syncthreads();
    long long my_store = 0, my_runs = 0;
    for (int k = 0; k < 2; ++k) {
        const int p = t + k * 1024;
        const unsigned long long kk = key[p];
        long long len = 0;
        if (kk != ~0ull) {
            const int i = (int)(kk & (kSlots - 1));
            const int32_t target = (int32_t)(kk >> 11);
            if (i < cut && d.idx[target] > d.idx[d.s_v[i]]) len = d.s_nt[i];
        }
        val[p] = len;
        my_store += len;
        my_runs += (kk != ~0ull && head[p]) ? 1 : 0;
    }
    red[t] = my_store;
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) { if (t < o) red[t] += red[t + o]; __syncthreads(); }
    const long long total_store = red[0];
    __syncthreads();
    red[t] = my_runs;
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) { if (t < o) red[t] += red[t + o]; __syncthreads(); }
    const long long total_runs = red[0];
    __syncthreads();
    if (t == 0 && (ctl->arena_used + total_store > d.arena_cap || (long long)ctl->blk_used + total_runs > (long long)d.blk_cap))
        overflow_sh = 1;
    __syncthreads();
    if (overflow_sh) cut = 0;          // nothing is committed; the host gives up on this form
    if (!overflow_sh) {
        segmented_scan_2048(val, flag, head);
        // the last position of a run knows the run's total: it takes the arena space and links the chunk
        for (int k = 0; k < 2; ++k) {
            const int p = t + k * 1024;
            const unsigned long long kk = key[p];
            if (kk == ~0ull) continue;
            const bool last = p == kSlots - 1 || key[p + 1] == ~0ull || (key[p + 1] >> 11) != (kk >> 11);
            if (!last) continue;
            const long long total = val[p];
            const int hp = hpos[p];
            long long base = -1;
            if (total > 0) {
                const int32_t target = (int32_t)(kk >> 11);
                base = (long long)atomicAdd((unsigned long long*)&ctl->arena_used, (unsigned long long)total);
                int32_t b = d.head[target];
                if (b < 0 || d.blk_count[b] == kDescPerBlock) {
                    const int32_t nb = atomicAdd(&ctl->blk_used, 1);
                    d.blk_next[nb] = b;
                    d.blk_count[nb] = 0;
                    d.head[target] = nb;
                    b = nb;
                }
                const int c = d.blk_count[b];
                d.blk_off[(long long)b * kDescPerBlock + c] = base;
                d.blk_len[(long long)b * kDescPerBlock + c] = (int32_t)total;
                d.blk_count[b] = c + 1;
            }
            run_base[hp] = base;
        }
        __syncthreads();
        long long my_work = 0;
        for (int k = 0; k < 2; ++k) {
            const int i = t + k * 1024;
            if (i >= cut) continue;
            my_work += d.s_nrec[i] + 1;
            if (!(d.s_best[i] >= 0 && d.s_score[i] > 0)) continue;
            const int32_t v = d.s_v[i], target = d.s_best[i];
            d.parent[v] = target;
            d.up[v] = target;
            atomicAdd((unsigned long long*)&d.dsum[target], (unsigned long long)d.s_dv[i]);
            const int p = pos_of_slot[i];
            const int hp = hpos[p];
            const long long len = d.idx[target] > d.idx[v] ? (long long)d.s_nt[i] : 0;
            if (len > 0) {
                d.s_store[i] = 1;
                d.s_chunk_off[i] = run_base[hp] + (val[p] - len);
            }
        }
        __syncthreads();               // run_base has been read; its memory now holds the work sum
        red[t] = my_work;
        __syncthreads();
        for (int o = 512; o > 0; o >>= 1) { if (t < o) red[t] += red[t + o]; __syncthreads(); }
    }
    // the round's vertices leave the slot table
    for (int k = 0; k < 2; ++k) {
        const int i = t + k * 1024;
        if (i < n_prepared) d.slot_of[d.s_v[i]] = -1;
    }
    if (t == 0) {
        ctl->last_cut = cut;
        ctl->rounds += 1;
        if (overflow_sh) {
            ctl->overflow = 1;
        } else {
            const long long work_round = red[0];
            if (ctl->pos + cut == d.M && cut > 0) ctl->work_at_last = ctl->work + work_round - (d.s_nrec[cut - 1] + 1);
            ctl->work += work_round;
            ctl->pos += cut;
            const int P = ctl->P;
            int next = cut == n_prepared ? 2 * P : 2 * cut + 16;
            if (next < 32) next = 32;
            if (next > kSlots) next = kSlots;
            ctl->P = next;
        }
    }
}

// Round step 4: the kept edge lists go from the round's scratch memory to their chunks.
__global__ __launch_bounds__(256) void keep_lists_kernel(DS d) {
    const int cut = d.ctl->last_cut;
    if (blockIdx.x < kSlots / 4) {                 // small slots, one wavefront each
        const int i = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
        if (i >= cut || !d.s_store[i] || d.s_class[i] != kClassSmall) return;
        const Rec* src = d.scand + (long long)i * kSmallRecords;
        Rec* dst = d.arena + d.s_chunk_off[i];
        const int nt = d.s_nt[i];
        for (int j = lane; j < nt; j += 64) dst[j] = src[j];
        return;
    }
    const int n_units = d.ctl->n_units;
    for (int u = blockIdx.x - kSlots / 4; u < n_units; u += gridDim.x - kSlots / 4) {
        const int i = d.unit_slot[u];
        if (i >= cut || !d.s_store[i]) continue;
        const int k = u - d.s_unit0[i];
        const int nt = d.s_nt[i];
        const Rec* src = d.cand + d.s_cand_off[i];
        Rec* dst = d.arena + d.s_chunk_off[i];
        const int j_end = (k + 1) * kUnit < nt ? (k + 1) * kUnit : nt;
        for (int j = k * kUnit + (int)threadIdx.x; j < j_end; j += 256) dst[j] = src[j];
    }
}

}  // namespace

int build_dendrogram_on_device(const DeviceGraph& g, double work_budget, std::vector<int32_t>& parent,
                               std::vector<int32_t>& order, double* work_ratio, int64_t* rounds_out) {
    const int64_t M = g.M, two_m = g.two_m;
    parent.assign(M, -1);
    order.resize(M);
    if (work_ratio) *work_ratio = 0.0;
    if (rounds_out) *rounds_out = 0;
    if (M == 0) return kDendrogramDone;
    if (two_m >= ((int64_t)1 << 31)) return kDendrogramUseHost;

    Scratch tmp;
    DevBuf<int32_t> d_order, d_idx, d_parent, d_up, d_head, d_slot_of;
    DevBuf<long long> d_dsum;
    d_order.alloc(M); d_idx.alloc(M); d_parent.alloc(M); d_up.alloc(M); d_head.alloc(M); d_slot_of.alloc(M);
    d_dsum.alloc(M);
    {   // visiting order: stable sort of the ids by degree
        DevBuf<uint32_t> key, key_sorted;
        DevBuf<int32_t> id;
        key.alloc(M); key_sorted.alloc(M); id.alloc(M);
        hipLaunchKernelGGL(degree_keys_kernel, dim3(blocks_for(M, 256)), dim3(256), 0, 0, (long long)M,
                           reinterpret_cast<const long long*>(g.ptr.p), key.p, id.p);
        size_t bytes = 0;
        ACC_HIP(rocprim::radix_sort_pairs(nullptr, bytes, key.p, key_sorted.p, id.p, d_order.p, (size_t)M, 0u, 32u));
        ACC_HIP(rocprim::radix_sort_pairs(tmp.get(bytes), bytes, key.p, key_sorted.p, id.p, d_order.p, (size_t)M, 0u, 32u));
    }
    hipLaunchKernelGGL(init_state_kernel, dim3(blocks_for(M, 256)), dim3(256), 0, 0, (long long)M,
                       reinterpret_cast<const long long*>(g.ptr.p), d_order.p, d_idx.p, d_parent.p, d_up.p, d_dsum.p,
                       d_head.p, d_slot_of.p);
    ACC_HIP(hipGetLastError());

    // memory pools
    const int64_t blk_cap = M + 16;
    const int64_t arena_cap = 3 * two_m + M + 1024;
    const int64_t cand_cap = two_m + 1024;
    const int64_t desc_cap = M + 16;
    const int64_t unit_cap = two_m / kUnit + kSlots + 16;
    const int n_dense = (int)std::max<int64_t>(1, std::min<int64_t>(kMaxDense, ((int64_t)4 << 30) / (4 * M)));
    DevBuf<int32_t> blk_next, blk_count, blk_len, d_len, unit_slot, u_best, row_dirty, sI[11];
    DevBuf<long long> blk_off, d_off, d_start, u_score, u_second, sL[5];
    DevBuf<Rec> arena, scand, cand;
    DevBuf<uint32_t> bits, dense;
    DevBuf<Ctl> ctl;
    blk_next.alloc(blk_cap); blk_count.alloc(blk_cap);
    blk_off.alloc(blk_cap * kDescPerBlock); blk_len.alloc(blk_cap * kDescPerBlock);
    arena.alloc(arena_cap);
    scand.alloc((size_t)kSlots * kSmallRecords);
    cand.alloc(cand_cap);
    d_off.alloc(desc_cap); d_len.alloc(desc_cap); d_start.alloc(desc_cap);
    unit_slot.alloc(unit_cap); u_best.alloc(unit_cap); u_score.alloc(unit_cap); u_second.alloc(unit_cap);
    bits.alloc((size_t)kSlots * kRowWords);
    row_dirty.alloc(kSlots);
    dense.alloc((size_t)n_dense * (size_t)M);
    for (auto& b : sI) b.alloc(kSlots);
    for (auto& b : sL) b.alloc(kSlots);
    ctl.alloc(1);
    ACC_HIP(hipMemset(bits.p, 0, sizeof(uint32_t) * kSlots * kRowWords));
    ACC_HIP(hipMemset(row_dirty.p, 0, sizeof(int32_t) * kSlots));
    ACC_HIP(hipMemset(dense.p, 0, sizeof(uint32_t) * (size_t)n_dense * (size_t)M));
    Ctl h{};
    h.P = kSlots;
    ACC_HIP(hipMemcpy(ctl.p, &h, sizeof(Ctl), hipMemcpyHostToDevice));

    DS d{};
    d.M = M; d.two_m = two_m;
    d.gptr = reinterpret_cast<const long long*>(g.ptr.p); d.gadj = g.adj.p; d.order = d_order.p; d.idx = d_idx.p;
    d.parent = d_parent.p; d.up = d_up.p; d.dsum = d_dsum.p; d.head = d_head.p;
    d.blk_next = blk_next.p; d.blk_count = blk_count.p; d.blk_off = blk_off.p; d.blk_len = blk_len.p; d.blk_cap = (int32_t)blk_cap;
    d.arena = arena.p; d.arena_cap = arena_cap; d.ctl = ctl.p; d.slot_of = d_slot_of.p;
    d.s_v = sI[0].p; d.s_nrec = sI[1].p; d.s_class = sI[2].p; d.s_dense = sI[3].p; d.s_desc_off = sI[4].p; d.s_ndesc = sI[5].p;
    d.s_unit0 = sI[6].p; d.s_nunits = sI[7].p; d.s_nt = sI[8].p; d.s_best = sI[9].p; d.s_store = sI[10].p;
    d.s_cand_off = sL[0].p; d.s_score = sL[1].p; d.s_second = sL[2].p; d.s_dv = sL[3].p; d.s_chunk_off = sL[4].p;
    d.bits = bits.p; d.row_dirty = row_dirty.p; d.scand = scand.p; d.cand = cand.p; d.cand_cap = cand_cap;
    d.d_off = d_off.p; d.d_len = d_len.p; d.d_start = d_start.p; d.desc_cap = (int32_t)desc_cap;
    d.unit_slot = unit_slot.p; d.unit_cap = (int32_t)unit_cap; d.u_best = u_best.p; d.u_score = u_score.p; d.u_second = u_second.p;
    d.dense = dense.p; d.n_dense = n_dense;

    const int64_t graph_size = two_m + M;
    const int64_t work_limit = work_budget > 0 ? (int64_t)(work_budget * (double)graph_size) : 0;
    // Rounds are enqueued in groups without waiting; the control block is read back after each group.
    int group = 4;
    int status = -1;
    const int64_t max_groups = 4 * M + 64;     // every round advances by at least one vertex
    for (int64_t gi = 0; gi < max_groups && status < 0; ++gi) {
        for (int r = 0; r < group; ++r) {
            hipLaunchKernelGGL(prepare_round_kernel, dim3(1), dim3(1024), 0, 0, d);
            hipLaunchKernelGGL(decide_small_kernel, dim3(kSlots), dim3(64), 0, 0, d);
            hipLaunchKernelGGL(accumulate_large_kernel, dim3(kLargeBlocks), dim3(256), 0, 0, d);
            hipLaunchKernelGGL(score_large_kernel, dim3(kLargeBlocks), dim3(256), 0, 0, d);
            hipLaunchKernelGGL(commit_round_kernel, dim3(1), dim3(1024), 0, 0, d);
            hipLaunchKernelGGL(keep_lists_kernel, dim3(kSlots / 4 + kLargeBlocks), dim3(256), 0, 0, d);
        }
        hipLaunchKernelGGL(compress_paths_kernel, dim3(blocks_for(M, 256)), dim3(256), 0, 0, (long long)M, d_up.p);
        ACC_HIP(hipGetLastError());
        ACC_HIP(hipMemcpy(&h, ctl.p, sizeof(Ctl), hipMemcpyDeviceToHost));
        if (h.overflow) status = kDendrogramUseHost;
        else if (h.pos >= M) {
            status = (work_limit > 0 && h.work_at_last > work_limit) ? kDendrogramOverBudget : kDendrogramDone;
        } else if (work_limit > 0 && h.work > work_limit) status = kDendrogramOverBudget;
        else if (h.rounds >= 65536 && h.pos / h.rounds < 4 && (M - h.pos) > 262144) status = kDendrogramUseHost;   // crawling
        if (group < 64) group *= 2;
    }
    if (status < 0) status = kDendrogramUseHost;
    if (work_ratio) *work_ratio = graph_size ? (double)h.work / (double)graph_size : 0.0;
    if (rounds_out) *rounds_out = h.rounds;
    if (status == kDendrogramDone) {
        ACC_HIP(hipMemcpy(parent.data(), d_parent.p, sizeof(int32_t) * M, hipMemcpyDeviceToHost));
        ACC_HIP(hipMemcpy(order.data(), d_order.p, sizeof(int32_t) * M, hipMemcpyDeviceToHost));
        // consistency of the merge forest: a vertex joins either a vertex whose turn comes later or one
        // that had its turn and stayed a root; anything else is not a dendrogram of this procedure
        std::vector<int32_t> turn(M);
        for (int64_t k = 0; k < M; ++k) turn[order[k]] = (int32_t)k;
        for (int64_t v = 0; v < M; ++v) {
            const int32_t p = parent[v];
            if (p < 0) continue;
            if (p >= M || p == v || !(turn[p] > turn[v] || parent[p] < 0)) return kDendrogramUseHost;
        }
    }
    return status;
}

}  // namespace accspmm
