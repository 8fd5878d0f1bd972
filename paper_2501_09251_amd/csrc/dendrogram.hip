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
// that costs a round, never the result.  (Re-examining such slots exactly, every candidate's score
// with the degree the earlier slots add to it, was tried: 6 % fewer rounds on a 2^23-vertex R-MAT
// graph, but the re-examination cost more than the rounds it saved.)
//
// A community's edge list, as of its vertex's turn, is its own adjacency plus the lists of the
// vertices merged into it (each a list of (community, weight) pairs as of that vertex's turn);
// endpoints are mapped to their present roots when the list is read.  The lists of the vertices
// that one round merges into one target are stored as one chunk; a target's chunks are found
// through a chain of small directory blocks.
#include <algorithm>
#include <chrono>

#include "device_util.h"

namespace accspmm {
namespace {

using namespace detail;

constexpr int kSlots = 2048;          // most vertices decided per round
constexpr int kRowWords = kSlots / 32;
constexpr int kSmallRecords = 512;    // a slot with at most this many edge records is decided by one wavefront
constexpr int kHashSize = 1024;       // entries of that wavefront's hash table in LDS
constexpr int kUnit = 512;            // edge records per thread block for larger slots
constexpr int kLargeBlocks = 2048;    // grid of the kernels that walk those units
constexpr int kMaxDense = 64;         // larger slots per round (each owns a weight array over all vertices)
// Edge records of larger slots walked per round, the round's first larger slot aside.  Late in the order
// the slots are hubs with long lists that are each other's neighbours: few of them stand per round, and the
// ones behind would be walked again round after round.  Measured on a 2^23-vertex R-MAT graph (rounds, seconds):
// no budget 35.3 K, 2.86; 1 M 35.3 K, 2.83; 256 K 35.4 K, 2.63; 64 K 35.5 K, 2.39; 32 K 37.2 K, 2.40; 16 K 47.6 K, 2.75.
constexpr long long kRoundRecords = 65536;
// A target's chunks are listed in directory blocks inside one pool of 32-bit words.  A block is
// {next block or -1, descriptors in use, capacity, position of its first chunk} followed by
// `capacity` descriptors of four words (chunk offset low, high, length, position).  A chunk's
// position is the number of records in the target's earlier chunks: the target's list is its
// adjacency followed by its chunks in that order, and a record of it is found by walking to the
// block and bisecting the block's positions, so nothing has to be laid out again per round.  A
// target's first block holds 4 descriptors, each further one twice as many up to 1024 (a hub
// collects thousands of chunks; its chain stays a few dozen blocks long), and the newest block
// heads the chain.
// Blocks are referred to by their word offset divided by 4 (all block sizes are multiples of 4).
constexpr int kDirHeader = 4, kDirDesc = 4, kDirFirstCap = 4, kDirMaxCap = 1024;

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
    int overflow;            // a memory pool was exhausted: nothing more is committed
    long long dir_used;      // words of the directory pool in use
    int keep_units, pad;     // units of the round whose kept lists are still to be copied
    long long large_slots;   // larger slots prepared so far (a statistic)
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
    int32_t* head;        // per vertex: its newest directory block, -1 if none
    int32_t* tot_rec;     // per vertex: records in all its chunks
    int32_t* dir;         // the directory pool
    long long dir_cap;    // its size in words
    Rec* arena;
    long long arena_cap;
    Ctl* ctl;
    int32_t* slot_of;
    int32_t *s_v, *s_nrec, *s_class, *s_dense, *s_unit0, *s_nunits, *s_nt, *s_best, *s_store;
    long long *s_cand_off, *s_score, *s_second, *s_dv, *s_chunk_off;
    uint32_t* bits;
    int32_t* row_dirty;
    Rec* scand;
    Rec* cand;
    long long cand_cap;
    long long round_records;   // most edge records of larger slots walked per round (the first such slot aside)
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
                                  int32_t* slot_of, int32_t* tot_rec) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M) return;
    idx[order[i]] = (int32_t)i;
    parent[i] = -1;
    up[i] = (int32_t)i;
    dsum[i] = gptr[i + 1] - gptr[i];
    head[i] = -1;
    slot_of[i] = -1;
    tot_rec[i] = 0;
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

// exclusive prefix sum over the block's T threads; `total` gets the sum (sh: 16 entries)
template <int T>
__device__ __forceinline__ long long block_scan(long long x, long long* sh, long long& total) {
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    long long incl = x;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const long long y = __shfl_up(incl, o);
        if (lane >= o) incl += y;
    }
    if (lane == 63) sh[wave] = incl;
    __syncthreads();
    long long before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < T / 64; ++w) {
        const long long y = sh[w];
        if (w < wave) before += y;
        all += y;
    }
    total = all;
    __syncthreads();
    return before + incl - x;
}

// Round step 1 (one block of T threads, two consecutive slots per thread; a round has at most 2 T
// slots, so the small block serves the small rounds that make up most of the procedure): the round's vertices,
// the size of their edge lists, and, in slot order, the memory the larger slots need; then, one
// wavefront per larger slot, the slot's work units.
template <int T>
__device__ __forceinline__ void prepare_round(const DS& d) {
    __shared__ long long sh[16];
    __shared__ int first_unfit, n_large;
    __shared__ int large_list[kMaxDense];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    Ctl* const ctl = d.ctl;
    const long long pos = ctl->pos;
    const int P = ctl->P < 2 * T ? ctl->P : 2 * T;
    const int n = (int)(d.M - pos < (long long)P ? d.M - pos : (long long)P);
    if (t == 0) { first_unfit = n; n_large = 0; }
    int v[2], nrec[2], cls[2];
    for (int k = 0; k < 2; ++k) {
        const int i = 2 * t + k;
        v[k] = -1; nrec[k] = 0; cls[k] = kClassNone;
        if (i >= n) continue;
        const int32_t x = d.order[pos + i];
        v[k] = x;
        d.slot_of[x] = i;
        d.s_v[i] = x;
        const long long records = d.gptr[x + 1] - d.gptr[x] + d.tot_rec[x];
        nrec[k] = (int)records;
        cls[k] = records <= kSmallRecords ? kClassSmall : kClassLarge;
    }
    // what the larger slots need, as exclusive prefix sums in slot order
    auto need = [&](int k, int what) -> long long {
        if (cls[k] != kClassLarge) return 0;
        switch (what) {
            case 0: return 1;
            case 1: return nrec[k];
            default: return (nrec[k] + kUnit - 1) / kUnit;
        }
    };
    long long pre[3][2], tot[3];
    for (int what = 0; what < 3; ++what) {
        const long long a = need(0, what), b = need(1, what);
        const long long ex = block_scan<T>(a + b, sh, tot[what]);
        pre[what][0] = ex;
        pre[what][1] = ex + a;
    }
    const long long cap[3] = {(long long)d.n_dense, d.cand_cap, (long long)d.unit_cap};
    for (int k = 0; k < 2; ++k) {
        const int i = 2 * t + k;
        if (i >= n) continue;
        bool fit = true;
        for (int what = 0; what < 3; ++what) fit = fit && pre[what][k] + need(k, what) <= cap[what];
        // long lists: no more records per round than the budget, beyond the round's first larger slot (the
        // slots behind a hub mostly fail the tests, and walking their lists again every round is the cost)
        fit = fit && (pre[1][k] == 0 || pre[1][k] + need(k, 1) <= d.round_records);
        if (!fit) atomicMin(&first_unfit, i);
    }
    __syncthreads();
    const int n_eval = first_unfit;
    for (int k = 0; k < 2; ++k) {
        const int i = 2 * t + k;
        if (i >= n) continue;
        if (i >= n_eval) cls[k] = kClassSkipped;
        d.s_class[i] = cls[k];
        d.s_nrec[i] = nrec[k];
        d.s_nt[i] = 0;
        d.s_store[i] = 0;
        if (cls[k] != kClassLarge) continue;
        const int nunits = (nrec[k] + kUnit - 1) / kUnit;
        d.s_dense[i] = (int)pre[0][k];
        d.s_cand_off[i] = pre[1][k];
        d.s_unit0[i] = (int)pre[2][k];
        d.s_nunits[i] = nunits;
        large_list[atomicAdd(&n_large, 1)] = i;
    }
    __syncthreads();
    if (t == 0) {
        ctl->n_prepared = n;
        ctl->n_eval = n_eval;
        ctl->large_slots += n_large;
    }
    // the work units of the larger slots, one wavefront per slot
    for (int q = wave; q < n_large; q += T / 64) {
        const int i = large_list[q];
        const int u0 = d.s_unit0[i], nu = d.s_nunits[i];
        for (int u = lane; u < nu; u += 64) d.unit_slot[u0 + u] = i;
    }
    // units of the decided slots only: those of the first slot that did not fit, and of all after it, are not walked
    long long my_units = 0;
    for (int k = 0; k < 2; ++k)
        if (cls[k] == kClassLarge) my_units += (nrec[k] + kUnit - 1) / kUnit;
    long long all_units;
    (void)block_scan<T>(my_units, sh, all_units);
    if (t == 0) ctl->n_units = (int)all_units;
}

// Round step 2 (blocks of 256 threads).  The first kSlots blocks decide one small slot each: the
// weights towards the neighbouring communities are summed in a hash table in LDS, and the block
// finds the best and the runner-up.  The other blocks walk the edge records of the larger slots,
// kUnit per block: summed per community in the same kind of table first (late in the procedure
// most records of a hub lead to a few large communities), then added to the slot's weight array
// over all vertices; the communities met for the first time go to the slot's candidate list.
__global__ __launch_bounds__(256) void decide_round_kernel(DS d) {
    __shared__ int32_t hkey[kHashSize];
    __shared__ uint32_t hval[kHashSize];
    __shared__ long long sh_s[4], sh_second[4];
    __shared__ int32_t sh_r[4];
    __shared__ int count_sh, dirty_sh;
    __shared__ long long sd_off[kSmallRecords];
    __shared__ int sd_len[kSmallRecords], sd_start[kSmallRecords + 1];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    int32_t self = -1;
    auto add = [&](int32_t to, uint32_t w) {
        const int32_t r = find_root(d.up, to);
        if (r == self) return;
        uint32_t h = ((uint32_t)r * 2654435761u) >> 22;   // 10 bits
        for (int probe = 0; probe < kHashSize; ++probe) {
            const int32_t k = atomicCAS(&hkey[h], -1, r);
            if (k == -1 || k == r) { atomicAdd(&hval[h], w); return; }
            h = (h + 1) & (kHashSize - 1);
        }
    };
    if (blockIdx.x < kSlots) {
        const int i = blockIdx.x;
        if (i >= d.ctl->n_eval || d.s_class[i] != kClassSmall) return;
        const int32_t v = d.s_v[i];
        self = v;
        for (int e = t; e < kHashSize; e += 256) { hkey[e] = -1; hval[e] = 0; }
        if (t == 0) { count_sh = 0; dirty_sh = 0; }
        __syncthreads();
        const long long gb = d.gptr[v], ge = d.gptr[v + 1];
        for (long long p = gb + t; p < ge; p += 256) add(d.gadj[p], 1u);
        // chunks: their descriptors are staged in LDS (a small slot has at most kSmallRecords of them),
        // then every thread takes records of the concatenated lists
        int nd = 0;
        long long guard = d.dir_cap / 4;
        for (int32_t b = d.head[v]; b >= 0 && guard > 0 && nd <= kSmallRecords; --guard) {
            const int32_t* blk = d.dir + (long long)b * 4;
            const int c = blk[1];
            for (int e = t; e < c && nd + e < kSmallRecords; e += 256) {
                const int32_t* w = blk + kDirHeader + kDirDesc * e;
                sd_off[nd + e] = (long long)(uint32_t)w[0] | ((long long)w[1] << 32);
                sd_len[nd + e] = w[2];
            }
            nd += c;
            b = blk[0];
        }
        if (nd > kSmallRecords) nd = kSmallRecords;
        __syncthreads();
        if (t == 0) {
            int acc = 0;
            for (int e = 0; e < nd; ++e) { sd_start[e] = acc; acc += sd_len[e]; }
            sd_start[nd] = acc;
        }
        __syncthreads();
        const int chunk_records = sd_start[nd];
        for (int q = t; q < chunk_records; q += 256) {
            int lo = 0, hi = nd - 1;          // last chunk that starts at or before q
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (sd_start[mid] <= q) lo = mid; else hi = mid - 1;
            }
            const Rec r = d.arena[sd_off[lo] + (q - sd_start[lo])];
            add(r.to, r.w);
        }
        __syncthreads();
        const long long dv = d.dsum[v];
        Best best{kNoScore, kNoScore, -1};
        Rec* const out = d.scand + (long long)i * kSmallRecords;
        for (int e = t; e < kHashSize; e += 256) {
            const int32_t r = hkey[e];
            if (r < 0) continue;
            const uint32_t w = hval[e];
            best_add(best, (long long)w * d.two_m - d.dsum[r] * dv, r);
            const int j = d.slot_of[r];
            if (j >= 0) { atomicOr(&d.bits[(long long)i * kRowWords + (j >> 5)], 1u << (j & 31)); dirty_sh = 1; }
            out[atomicAdd(&count_sh, 1)] = Rec{r, w};
        }
        best = best_wave_reduce(best);
        if (lane == 0) { sh_s[wave] = best.s; sh_second[wave] = best.second; sh_r[wave] = best.r; }
        __syncthreads();
        if (t == 0) {
            Best all{sh_s[0], sh_second[0], sh_r[0]};
            for (int w2 = 1; w2 < 4; ++w2) best_join(all, Best{sh_s[w2], sh_second[w2], sh_r[w2]});
            if (dirty_sh) d.row_dirty[i] = 1;
            d.s_nt[i] = count_sh;
            d.s_best[i] = all.r;
            d.s_score[i] = all.s;
            d.s_second[i] = all.second;
            d.s_dv[i] = dv;
        }
        return;
    }
    const int n_units = d.ctl->n_units;
    for (int u = blockIdx.x - kSlots; u < n_units; u += gridDim.x - kSlots) {
        const int i = d.unit_slot[u];
        const int k = u - d.s_unit0[i];
        self = d.s_v[i];
        const int nrec = d.s_nrec[i];
        const int32_t vtx = d.s_v[i];
        const long long adj0 = d.gptr[vtx];
        const int deg = (int)(d.gptr[vtx + 1] - adj0);
        const int32_t head_blk = d.head[vtx];
        uint32_t* const weight = d.dense + (long long)d.s_dense[i] * d.M;
        Rec* const cand = d.cand + d.s_cand_off[i];
        const int p_end = (k + 1) * kUnit < nrec ? (k + 1) * kUnit : nrec;
        for (int e = t; e < kHashSize; e += 256) { hkey[e] = -1; hval[e] = 0; }
        __syncthreads();
        for (int p = k * kUnit + t; p < p_end; p += 256) {
            if (p < deg) { add(d.gadj[adj0 + p], 1u); continue; }
            const int pc = p - deg;                       // position among the records of the chunks
            const int32_t* blk = d.dir + (long long)head_blk * 4;
            long long guard = d.dir_cap / 4;
            while (blk[3] > pc && blk[0] >= 0 && guard-- > 0) blk = d.dir + (long long)blk[0] * 4;   // newest block first
            int lo = 0, hi = blk[1] - 1;                  // last chunk of the block that starts at or before pc
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (blk[kDirHeader + kDirDesc * mid + 3] <= pc) lo = mid; else hi = mid - 1;
            }
            const int32_t* w = blk + kDirHeader + kDirDesc * lo;
            const Rec r = d.arena[((long long)(uint32_t)w[0] | ((long long)w[1] << 32)) + (pc - w[3])];
            add(r.to, r.w);
        }
        __syncthreads();
        for (int e = t; e < kHashSize; e += 256) {
            const int32_t r = hkey[e];
            if (r < 0) continue;
            if (atomicAdd(&weight[r], hval[e]) == 0u) cand[atomicAdd(&d.s_nt[i], 1)].to = r;
        }
        __syncthreads();
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

// ascending bitonic sort of the first n2 keys (a power of two, at most 2048) in LDS
template <int T>
__device__ __forceinline__ void bitonic_sort_lds(unsigned long long* key, int n2) {
    const int t = threadIdx.x;
    for (int size = 2; size <= n2; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int c = t; c < (n2 >> 1); c += T) {
                const int lo = ((c & ~(stride - 1)) << 1) | (c & (stride - 1));
                const int hi = lo + stride;
                const bool up = (lo & size) == 0;
                const unsigned long long a = key[lo], b = key[hi];
                if ((a > b) == up) { key[lo] = b; key[hi] = a; }
            }
        }
    }
    __syncthreads();
}

// inclusive sums of val inside runs (a run starts where head is set) over the first n2 positions
template <int T>
__device__ __forceinline__ void segmented_scan_lds(long long* val, uint8_t* flag, const uint8_t* head, int n2) {
    constexpr int kPer = kSlots / T;
    const int t = threadIdx.x;
    for (int p = t; p < n2; p += T) flag[p] = head[p];
    __syncthreads();
    for (int o = 1; o < n2; o <<= 1) {
        long long add[kPer];
        uint8_t f[kPer];
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            const int p = t + k * T;
            add[k] = 0;
            f[k] = 0;
            if (p >= n2) continue;
            f[k] = flag[p];
            if (p >= o && !flag[p]) { add[k] = val[p - o]; f[k] = flag[p - o]; }
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            const int p = t + k * T;
            if (p >= n2) continue;
            val[p] += add[k];
            flag[p] = f[k];
        }
        __syncthreads();
    }
}

template <int T>
__device__ __forceinline__ long long block_sum_commit(long long x, long long* sh16) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh16[threadIdx.x >> 6] = x;
    __syncthreads();
    long long all = 0;
#pragma unroll
    for (int w = 0; w < T / 64; ++w) all += sh16[w];
    return all;
}

constexpr int kQuadratic = 128;   // rounds of at most this many slots compare all pairs of slots instead of sorting

// Directory words that appending one more chunk to `target` takes: a new block where the target has
// none or its newest one is full.
__device__ __forceinline__ int dir_words_for_append(const DS& d, int32_t target) {
    const int32_t b = d.head[target];
    const int32_t* blk = b >= 0 ? d.dir + (long long)b * 4 : nullptr;
    if (blk && blk[1] < blk[2]) return 0;
    int cap = blk ? 2 * blk[2] : kDirFirstCap;
    if (cap > kDirMaxCap) cap = kDirMaxCap;
    return kDirHeader + kDirDesc * cap;
}

// Takes `total` records of the arena as a new chunk of `target` and lists it in the target's
// directory; returns the chunk's offset.  One thread per target and round calls this, after the
// round's needs were checked against the pools.
__device__ __forceinline__ long long append_chunk(const DS& d, int32_t target, long long total) {
    Ctl* const ctl = d.ctl;
    const long long base = (long long)atomicAdd((unsigned long long*)&ctl->arena_used, (unsigned long long)total);
    int32_t b = d.head[target];
    int32_t* blk = b >= 0 ? d.dir + (long long)b * 4 : nullptr;
    if (!blk || blk[1] == blk[2]) {
        int cap = blk ? 2 * blk[2] : kDirFirstCap;
        if (cap > kDirMaxCap) cap = kDirMaxCap;
        const long long at = (long long)atomicAdd((unsigned long long*)&ctl->dir_used, (unsigned long long)(kDirHeader + kDirDesc * cap));
        int32_t* nb = d.dir + at;
        nb[0] = b;
        nb[1] = 0;
        nb[2] = cap;
        nb[3] = d.tot_rec[target];       // position of the block's first chunk
        d.head[target] = (int32_t)(at >> 2);
        blk = nb;
    }
    const int c = blk[1];
    int32_t* w = blk + kDirHeader + kDirDesc * c;
    w[0] = (int32_t)(uint32_t)(base & 0xffffffffll);
    w[1] = (int32_t)(base >> 32);
    w[2] = (int32_t)total;
    w[3] = d.tot_rec[target];
    blk[1] = c + 1;
    d.tot_rec[target] += (int32_t)total;
    return base;
}

// Round step 3 (one block of T threads): which slots stand, and the commit of those.
//
// Merging slots are grouped by target, in slot order inside a group: the degree that earlier slots
// of the round add to a slot's target is a prefix sum inside its group (test (c)), and the lists
// that the committed slots of a group keep form one chunk, each list at its prefix offset.  Rounds of
// more than kQuadratic slots sort (target, slot) keys and scan the sorted runs.  Smaller rounds, the
// great majority, let every slot look at the slots before it directly, with a handful of barriers
// instead of a hundred.
template <int T>
__global__ __launch_bounds__(T) void commit_round_kernel(DS d) {
    constexpr int kPer = kSlots / T;
    __shared__ unsigned long long key[kSlots];
    __shared__ long long val[kSlots];
    __shared__ long long run_base[kSlots];       // arena offset of a group's chunk, at the group's first position
    __shared__ long long sh16[16];
    __shared__ uint32_t mmask[kRowWords];
    __shared__ uint8_t inv[kSlots], head[kSlots], flag[kSlots];
    __shared__ int16_t pos_of_slot[kSlots], hpos[kSlots];
    __shared__ int32_t tg[kQuadratic], want[kQuadratic];
    __shared__ int cut_sh, overflow_sh, n_large_sh;
    __shared__ int16_t large_list[kMaxDense];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    Ctl* const ctl = d.ctl;
    const int n_prepared = ctl->n_prepared, n_eval = ctl->n_eval;
    if (n_prepared == 0) {
        // a round enqueued after the last vertex had its turn: nothing was kept, and the next launch must
        // not copy the last real round's lists again from the other set of per-slot arrays
        if (t == 0) { ctl->last_cut = 0; ctl->keep_units = 0; }
        return;
    }
    const long long pos = ctl->pos;
    const bool direct = n_eval <= kQuadratic;
    int n2 = 64;
    while (n2 < n_eval) n2 <<= 1;
    if (t < kRowWords) mmask[t] = 0;
    if (t == 0) { cut_sh = n_eval; overflow_sh = 0; n_large_sh = 0; }
    for (int i = t; i < n2; i += T) { inv[i] = 0; flag[i] = i < n_eval ? (uint8_t)d.row_dirty[i] : (uint8_t)0; }
    __syncthreads();
    // a slot that merges: its key, its degree, and in a small round its target and what it keeps
    auto merging_slot = [&](int i) {
        const int32_t best = d.s_best[i];
        if (best >= 0 && d.s_score[i] > 0) {
            atomicOr(&mmask[i >> 5], 1u << (i & 31));
            key[i] = ((unsigned long long)(uint32_t)best << 11) | (unsigned long long)i;
            val[i] = d.s_dv[i];
            if (direct) {
                tg[i] = best;
                want[i] = (long long)d.idx[best] > pos + i ? d.s_nt[i] : 0;   // the list is kept if the target's turn is ahead
                const int s = d.slot_of[best];
                if (s > i && s < n_eval) inv[s] = 1;                          // (b), see below
            }
        }
    };
    // results of the larger slots from their blocks' partial results; who merges
    constexpr int kUnitsInline = 128;
    for (int i = t; i < n2; i += T) {
        key[i] = ~0ull;
        val[i] = 0;
        if (i < kQuadratic) { tg[i] = -1; want[i] = 0; }
        if (i >= n_eval) continue;
        if (d.s_class[i] == kClassLarge) {
            const int u0 = d.s_unit0[i], nu = d.s_nunits[i];
            if (nu > kUnitsInline) {      // a hub: left to a whole wavefront below
                large_list[atomicAdd(&n_large_sh, 1)] = (int16_t)i;    // at most kMaxDense larger slots per round
                continue;
            }
            Best all{kNoScore, kNoScore, -1};
            for (int u = u0; u < u0 + nu; ++u) best_join(all, Best{d.u_score[u], d.u_second[u], d.u_best[u]});
            d.s_best[i] = all.r;
            d.s_score[i] = all.s;
            d.s_second[i] = all.second;
            d.s_dv[i] = d.dsum[d.s_v[i]];
        }
        merging_slot(i);
    }
    __syncthreads();
    if (n_large_sh > 0) {     // hubs whose lists thousands of blocks walked: one wavefront reduces a slot's partial results
        for (int q = wave; q < n_large_sh; q += T / 64) {
            const int i = large_list[q];
            Best all{kNoScore, kNoScore, -1};
            const int u0 = d.s_unit0[i], nu = d.s_nunits[i];
            for (int u = u0 + lane; u < u0 + nu; u += 64) best_join(all, Best{d.u_score[u], d.u_second[u], d.u_best[u]});
            all = best_wave_reduce(all);
            if (lane == 0) {
                d.s_best[i] = all.r;
                d.s_score[i] = all.s;
                d.s_second[i] = all.second;
                d.s_dv[i] = d.dsum[d.s_v[i]];
                __threadfence_block();
                merging_slot(i);
            }
        }
        __syncthreads();
    }
    // (b) an earlier slot merges into this slot's vertex
    if (!direct)
        for (int j = t; j < n_eval; j += T) {
            if (key[j] == ~0ull) continue;
            const int s = d.slot_of[d.s_best[j]];
            if (s > j && s < n_eval) inv[s] = 1;
        }
    // (a) a candidate community is the vertex of an earlier slot that merges
    for (int i = wave; i < n_eval; i += T / 64) {
        if (!flag[i]) continue;
        const uint32_t word = d.bits[(long long)i * kRowWords + lane];
        const uint32_t below = lane < (i >> 5) ? 0xffffffffu : (lane == (i >> 5) ? ((1u << (i & 31)) - 1u) : 0u);
        if (__ballot((word & mmask[lane] & below) != 0u) && lane == 0) inv[i] = 1;
        d.bits[(long long)i * kRowWords + lane] = 0u;
        if (lane == 0) d.row_dirty[i] = 0;
    }
    long long work_round = 0;
    int cut;
    if (direct) {
        // ---- small round: slot i looks at the slots before it
        long long offset_in_chunk = 0;     // records that earlier slots of the group keep
        int first = -1;                    // the group's first slot
        int32_t my_tg = -1;
        if (t < n_eval && (my_tg = tg[t]) >= 0) {
            long long before = 0;
            first = t;
#pragma unroll 8
            for (int j = 0; j < t; ++j) {
                const bool same = tg[j] == my_tg;
                before += same ? val[j] : 0;
                offset_in_chunk += same ? want[j] : 0;
                first = same && j < first ? j : first;
            }
            if (before > 0) {   // (c)
                const long long adjusted = d.s_score[t] - before * val[t];
                if (!(adjusted > 0 && adjusted > d.s_second[t])) inv[t] = 1;
            }
        }
        __syncthreads();
        if (t < n_eval && inv[t]) atomicMin(&cut_sh, t);
        __syncthreads();
        cut = cut_sh;
        // a group's first slot sums what the group's committed slots keep and takes the space
        long long total = 0;
        int words = 0;
        const bool leader = my_tg >= 0 && first == t && t < cut;
        if (leader) {
            for (int j = t; j < cut; ++j) total += tg[j] == my_tg ? want[j] : 0;
            if (total > 0) words = dir_words_for_append(d, my_tg);
        }
        const long long total_store = block_sum_commit<T>(total, sh16);
        const long long total_words = block_sum_commit<T>(words, sh16);
        if (t == 0 && (ctl->arena_used + total_store > d.arena_cap || ctl->dir_used + total_words > d.dir_cap)) overflow_sh = 1;
        __syncthreads();
        if (overflow_sh) cut = 0;
        if (leader && total > 0 && !overflow_sh) run_base[t] = append_chunk(d, my_tg, total);
        __syncthreads();
        long long my_work = 0;
        if (t < cut) {
            my_work = d.s_nrec[t] + 1;
            if (my_tg >= 0) {
                const int32_t v = d.s_v[t];
                d.parent[v] = my_tg;
                d.up[v] = my_tg;
                atomicAdd((unsigned long long*)&d.dsum[my_tg], (unsigned long long)val[t]);
                if (want[t] > 0) {
                    d.s_store[t] = 1;
                    d.s_chunk_off[t] = run_base[first] + offset_in_chunk;
                }
            }
        }
        work_round = block_sum_commit<T>(my_work, sh16);
    } else {
        // ---- large round: merging slots sorted by (target, slot)
        bitonic_sort_lds<T>(key, n2);
        for (int p = t; p < n2; p += T) {
            const unsigned long long kk = key[p];
            head[p] = p == 0 || (kk >> 11) != (key[p - 1] >> 11);
            val[p] = kk == ~0ull ? 0 : d.s_dv[(int)(kk & (kSlots - 1))];
            if (kk != ~0ull) pos_of_slot[(int)(kk & (kSlots - 1))] = (int16_t)p;
        }
        __syncthreads();
        // first position of every position's run: running maximum of the head positions
        for (int p = t; p < n2; p += T) hpos[p] = head[p] ? (int16_t)p : (int16_t)0;
        __syncthreads();
        for (int o = 1; o < n2; o <<= 1) {
            int16_t m[kPer];
#pragma unroll
            for (int k = 0; k < kPer; ++k) {
                const int p = t + k * T;
                m[k] = 0;
                if (p < n2) m[k] = p >= o && hpos[p - o] > hpos[p] ? hpos[p - o] : hpos[p];
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < kPer; ++k) if (t + k * T < n2) hpos[t + k * T] = m[k];
            __syncthreads();
        }
        segmented_scan_lds<T>(val, flag, head, n2);
        for (int p = t; p < n2; p += T) {     // (c)
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
        for (int i = t; i < n_eval; i += T)
            if (inv[i]) atomicMin(&cut_sh, i);
        __syncthreads();
        cut = cut_sh;
        // lists to keep: those of committed merges whose target has its turn still ahead; val becomes the
        // list's length and then the inclusive prefix of the lengths inside the run
        long long my_store = 0;
        for (int p = t; p < n2; p += T) {
            const unsigned long long kk = key[p];
            long long len = 0;
            if (kk != ~0ull) {
                const int i = (int)(kk & (kSlots - 1));
                if (i < cut && (long long)d.idx[(int32_t)(kk >> 11)] > pos + i) len = d.s_nt[i];
            }
            val[p] = len;
            my_store += len;
        }
        const long long total_store = block_sum_commit<T>(my_store, sh16);
        segmented_scan_lds<T>(val, flag, head, n2);
        // a run's last position holds the run's total: it takes the arena space and links the chunk
        auto last_of_run = [&](int p) { return p == n2 - 1 || key[p + 1] == ~0ull || (key[p + 1] >> 11) != (key[p] >> 11); };
        long long my_words = 0;
        for (int p = t; p < n2; p += T) {
            const unsigned long long kk = key[p];
            if (kk == ~0ull || val[p] == 0 || !last_of_run(p)) continue;
            my_words += dir_words_for_append(d, (int32_t)(kk >> 11));
        }
        const long long total_words = block_sum_commit<T>(my_words, sh16);
        if (t == 0 && (ctl->arena_used + total_store > d.arena_cap || ctl->dir_used + total_words > d.dir_cap)) overflow_sh = 1;
        __syncthreads();
        if (overflow_sh) cut = 0;          // nothing is committed; the host gives up on this form
        if (!overflow_sh) {
            for (int p = t; p < n2; p += T) {
                const unsigned long long kk = key[p];
                if (kk == ~0ull || val[p] == 0 || !last_of_run(p)) continue;
                run_base[hpos[p]] = append_chunk(d, (int32_t)(kk >> 11), val[p]);
            }
            __syncthreads();
            long long my_work = 0;
            for (int i = t; i < cut; i += T) {
                my_work += d.s_nrec[i] + 1;
                if (!(d.s_best[i] >= 0 && d.s_score[i] > 0)) continue;
                const int32_t v = d.s_v[i], target = d.s_best[i];
                d.parent[v] = target;
                d.up[v] = target;
                atomicAdd((unsigned long long*)&d.dsum[target], (unsigned long long)d.s_dv[i]);
                const int p = pos_of_slot[i];
                const long long len = (long long)d.idx[target] > pos + i ? (long long)d.s_nt[i] : 0;
                if (len > 0) {
                    d.s_store[i] = 1;
                    d.s_chunk_off[i] = run_base[hpos[p]] + (val[p] - len);
                }
            }
            work_round = block_sum_commit<T>(my_work, sh16);
        }
    }
    // the round's vertices leave the slot table
    for (int i = t; i < n_prepared; i += T) d.slot_of[d.s_v[i]] = -1;
    if (t == 0) {
        ctl->last_cut = cut;
        ctl->keep_units = ctl->n_units;
        ctl->rounds += 1;
        if (overflow_sh) {
            ctl->overflow = 1;
        } else {
            if (pos + cut == d.M && cut > 0) ctl->work_at_last = ctl->work + work_round - (d.s_nrec[cut - 1] + 1);
            ctl->work += work_round;
            ctl->pos = pos + cut;
            const int P = ctl->P;
            int next = cut == n_prepared ? 2 * P : 2 * cut + 16;
            if (next < 32) next = 32;
            if (next > kSlots) next = kSlots;
            ctl->P = next;
        }
    }
}

// Round step 4: the kept edge lists go from the round's scratch memory to their chunks.  Runs in the
// blocks after the first of the next round's prepare launch (kKeepBlocks blocks of any size): the
// per-slot arrays and the unit table exist twice and alternate between rounds, so the next round's
// preparation does not overwrite what this reads.
constexpr int kKeepBlocks = 256;
__device__ __forceinline__ void keep_lists(const DS& d, int b, int nthreads) {
    const int cut = d.ctl->last_cut;
    const int waves = nthreads / 64, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int i = b * waves + wave; i < cut; i += kKeepBlocks * waves) {      // small slots, one wavefront each
        if (!d.s_store[i] || d.s_class[i] != kClassSmall) continue;
        const Rec* src = d.scand + (long long)i * kSmallRecords;
        Rec* dst = d.arena + d.s_chunk_off[i];
        const int nt = d.s_nt[i];
        for (int j = lane; j < nt; j += 64) dst[j] = src[j];
    }
    const int n_units = d.ctl->keep_units;
    for (int u = b; u < n_units; u += kKeepBlocks) {
        const int i = d.unit_slot[u];
        if (i < 0 || i >= cut || !d.s_store[i]) continue;
        const int k = u - d.s_unit0[i];
        const int nt = d.s_nt[i];
        const Rec* src = d.cand + d.s_cand_off[i];
        Rec* dst = d.arena + d.s_chunk_off[i];
        const int j_end = (k + 1) * kUnit < nt ? (k + 1) * kUnit : nt;
        for (int j = k * kUnit + (int)threadIdx.x; j < j_end; j += nthreads) dst[j] = src[j];
    }
}

template <int T>
__global__ __launch_bounds__(T) void prepare_and_keep_kernel(DS cur, DS prev) {
    if (blockIdx.x == 0) prepare_round<T>(cur);
    else keep_lists(prev, (int)blockIdx.x - 1, T);
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
    DevBuf<int32_t> d_order, d_idx, d_parent, d_up, d_head, d_slot_of, d_tot_rec;
    DevBuf<long long> d_dsum;
    d_order.alloc(M); d_idx.alloc(M); d_parent.alloc(M); d_up.alloc(M); d_head.alloc(M); d_slot_of.alloc(M);
    d_tot_rec.alloc(M);
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
                       d_head.p, d_slot_of.p, d_tot_rec.p);
    ACC_HIP(hipGetLastError());

    // memory pools
    // words: a first block per target (16 words); every further block doubles, so a target's blocks hold
    // at most twice its chunks (3 words each) plus headers; targets and chunks are at most M each
    const int64_t dir_cap = 36 * M + 8192;
    // list lengths are 32-bit: a vertex's records are its adjacency (fewer than M) plus what lies in the
    // arena, so an arena of fewer than 2^31 - M records keeps every length in range (a graph that needs
    // more exhausts the pool and goes to the host form)
    const int64_t arena_cap = std::min<int64_t>(3 * two_m + M + 1024, ((int64_t)1 << 31) - M - 1024);
    const int64_t cand_cap = two_m + 1024;
    const int64_t unit_cap = two_m / kUnit + kSlots + 16;
    const int n_dense = (int)std::max<int64_t>(1, std::min<int64_t>(kMaxDense, ((int64_t)4 << 30) / (4 * M)));
    DevBuf<int32_t> dir, unit_slot, u_best, row_dirty, sI[9];
    DevBuf<long long> u_score, u_second, sL[5];
    DevBuf<Rec> arena, scand, cand;
    DevBuf<uint32_t> bits, dense;
    DevBuf<Ctl> ctl;
    dir.alloc(dir_cap);
    arena.alloc(arena_cap);
    scand.alloc((size_t)kSlots * kSmallRecords);
    cand.alloc(cand_cap);
    unit_slot.alloc(2 * unit_cap); u_best.alloc(unit_cap); u_score.alloc(unit_cap); u_second.alloc(unit_cap);
    bits.alloc((size_t)kSlots * kRowWords);
    row_dirty.alloc(kSlots);
    dense.alloc((size_t)n_dense * (size_t)M);
    for (auto& b : sI) b.alloc(2 * kSlots);      // two sets, alternating between rounds
    for (auto& b : sL) b.alloc(2 * kSlots);
    ctl.alloc(1);
    ACC_HIP(hipMemset(bits.p, 0, sizeof(uint32_t) * kSlots * kRowWords));
    ACC_HIP(hipMemset(row_dirty.p, 0, sizeof(int32_t) * kSlots));
    ACC_HIP(hipMemset(unit_slot.p, 0, sizeof(int32_t) * 2 * (size_t)unit_cap));
    for (auto& b : sI) ACC_HIP(hipMemset(b.p, 0, sizeof(int32_t) * 2 * kSlots));
    for (auto& b : sL) ACC_HIP(hipMemset(b.p, 0, sizeof(long long) * 2 * kSlots));
    ACC_HIP(hipMemset(dense.p, 0, sizeof(uint32_t) * (size_t)n_dense * (size_t)M));
    Ctl h{};
    h.P = kSlots;
    ACC_HIP(hipMemcpy(ctl.p, &h, sizeof(Ctl), hipMemcpyHostToDevice));

    DS d{};
    d.M = M; d.two_m = two_m;
    d.gptr = reinterpret_cast<const long long*>(g.ptr.p); d.gadj = g.adj.p; d.order = d_order.p; d.idx = d_idx.p;
    d.parent = d_parent.p; d.up = d_up.p; d.dsum = d_dsum.p; d.head = d_head.p;
    d.tot_rec = d_tot_rec.p;
    d.dir = dir.p; d.dir_cap = dir_cap;
    d.round_records = kRoundRecords;
    d.arena = arena.p; d.arena_cap = arena_cap; d.ctl = ctl.p; d.slot_of = d_slot_of.p;
    d.s_v = sI[0].p; d.s_nrec = sI[1].p; d.s_class = sI[2].p; d.s_dense = sI[3].p;
    d.s_unit0 = sI[4].p; d.s_nunits = sI[5].p; d.s_nt = sI[6].p; d.s_best = sI[7].p; d.s_store = sI[8].p;
    d.s_cand_off = sL[0].p; d.s_score = sL[1].p; d.s_second = sL[2].p; d.s_dv = sL[3].p; d.s_chunk_off = sL[4].p;
    d.bits = bits.p; d.row_dirty = row_dirty.p; d.scand = scand.p; d.cand = cand.p; d.cand_cap = cand_cap;
    d.unit_slot = unit_slot.p; d.unit_cap = (int32_t)unit_cap; d.u_best = u_best.p; d.u_score = u_score.p; d.u_second = u_second.p;
    d.dense = dense.p; d.n_dense = n_dense;

    // the second set of per-slot arrays and unit table
    DS d_odd = d;
    {
        int32_t** ip[] = {&d_odd.s_v, &d_odd.s_nrec, &d_odd.s_class, &d_odd.s_dense,
                          &d_odd.s_unit0, &d_odd.s_nunits, &d_odd.s_nt, &d_odd.s_best, &d_odd.s_store};
        for (auto pp : ip) *pp += kSlots;
        long long** lp[] = {&d_odd.s_cand_off, &d_odd.s_score, &d_odd.s_second, &d_odd.s_dv, &d_odd.s_chunk_off};
        for (auto pp : lp) *pp += kSlots;
        d_odd.unit_slot += unit_cap;
    }
    const int64_t graph_size = two_m + M;
    const int64_t work_limit = work_budget > 0 ? (int64_t)(work_budget * (double)graph_size) : 0;
    // Rounds are enqueued in groups without waiting; the control block is read back after each group.
    int group = 4;
    int status = -1;
    long long rounds_before = 0, pos_before = 0, launched = 0;
    // what the sequential host form needs for the whole graph, roughly (it measured 19 ns per graph entry on
    // 500 M entries and less on graphs that fit the caches), and the least time worth a change of form
    const double host_estimate_s = std::max(25e-9 * (double)graph_size, 0.25);
    const int64_t max_groups = 4 * M + 64;     // every round advances by at least one vertex
    for (int64_t gi = 0; gi < max_groups && status < 0; ++gi) {
        // block sizes follow what the last group of rounds looked like: large rounds sort in the commit
        // kernel; the preparation handles two slots per thread
        const bool wide = h.P > kQuadratic;
        const bool wide_prepare = h.P > 512;
        rounds_before = h.rounds;
        pos_before = h.pos;
        const auto group_start = std::chrono::steady_clock::now();
        for (int r = 0; r < group; ++r, ++launched) {
            const DS& cur = (launched & 1) ? d_odd : d;
            const DS& prev = (launched & 1) ? d : d_odd;
            // this round's preparation, and beside it the copy of the lists the last round kept
            if (wide_prepare) hipLaunchKernelGGL(prepare_and_keep_kernel<1024>, dim3(1 + kKeepBlocks), dim3(1024), 0, 0, cur, prev);
            else hipLaunchKernelGGL(prepare_and_keep_kernel<256>, dim3(1 + kKeepBlocks), dim3(256), 0, 0, cur, prev);
            hipLaunchKernelGGL(decide_round_kernel, dim3(kSlots + kLargeBlocks), dim3(256), 0, 0, cur);
            hipLaunchKernelGGL(score_large_kernel, dim3(kLargeBlocks), dim3(256), 0, 0, cur);
            if (wide) hipLaunchKernelGGL(commit_round_kernel<1024>, dim3(1), dim3(1024), 0, 0, cur);
            else hipLaunchKernelGGL(commit_round_kernel<256>, dim3(1), dim3(256), 0, 0, cur);
        }
        hipLaunchKernelGGL(compress_paths_kernel, dim3(blocks_for(M, 256)), dim3(256), 0, 0, (long long)M, d_up.p);
        ACC_HIP(hipGetLastError());
        ACC_HIP(hipMemcpy(&h, ctl.p, sizeof(Ctl), hipMemcpyDeviceToHost));
        if (h.overflow) status = kDendrogramUseHost;
        else if (h.pos >= M) {
            status = (work_limit > 0 && h.work_at_last > work_limit) ? kDendrogramOverBudget : kDendrogramDone;
        } else if (work_limit > 0 && h.work > work_limit) status = kDendrogramOverBudget;
        else if (h.rounds >= 256) {
            // crawling: at the pace of the last group of rounds the rest would take longer than the host form
            // needs for everything (chains of vertices that each depend on the one before, as in banded
            // matrices, where a round commits one or two vertices)
            const double group_s = std::chrono::duration<double>(std::chrono::steady_clock::now() - group_start).count();
            const double group_rounds = (double)std::max<long long>(1, h.rounds - rounds_before);
            const double per_round = (double)(h.pos - pos_before) / group_rounds;
            const double rest_s = (double)(M - h.pos) / std::max(per_round, 1e-3) * (group_s / group_rounds);
            if (rest_s > host_estimate_s) status = kDendrogramUseHost;
        }
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
