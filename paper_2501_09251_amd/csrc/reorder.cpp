// Data-affinity-based row reordering (paper Section 3.2, Algorithm 1), host side.
//
// Step I (dendrogram construction) is sequential by definition: vertices are visited in
// ascending degree and every decision depends on the merges made before it, so it runs on
// one host thread over flat arrays.  The graph it reads is built on the GPU (graph.hip);
// this file ends with the dendrogram's leaf sequence cut into segments; Step II (ordering
// generation), which is independent per segment, runs on the GPU again (ordering.hip).
//
// Readings of what the paper leaves open (Eq. 1 is printed as the modularity itself, the
// tie-breaks and the search scope of Step II are not stated):
//  - graph: vertex per row/column index, undirected unit edge {i,j}, i != j, iff A_ij or
//    A_ji is stored;
//  - visiting order: ascending degree, ties by lower id;
//  - gain of joining communities u and v: 2*(w_uv/(2m) - d_u*d_v/(2m)^2), compared exactly
//    as s = w_uv*2m - d_u*d_v in 64-bit integers; ties go to the lower community id; merge
//    only when s > 0;
//  - leaf sequence: roots by ascending id, a root first and then its children's subtrees
//    in merge order; every tree's sequence is cut into segments of at most seg_len leaves;
//  - chaining inside a segment: next is the unvisited leaf sharing the most column indices
//    with the current row (at least one), ties to the earliest leaf of the sequence.
#include <algorithm>
#include <memory>

#include "internal.h"

namespace accspmm {
namespace {

struct Edge {
    int32_t to;
    uint32_t w;
};

// Recycling allocator for the per-community edge lists of Step I.  Lists live from a
// vertex's turn to its parent's turn; handing their blocks (power-of-two sizes) back for
// reuse keeps the loop on memory that is already mapped and warm, instead of taking a
// first-touch page fault for every new list.
class EdgeArena {
public:
    static int size_class(size_t n) {
        int c = 3;
        while (((size_t)1 << c) < n) ++c;
        return c;
    }
    Edge* take(int cls) {
        auto& fl = free_[cls];
        if (!fl.empty()) {
            Edge* p = fl.back();
            fl.pop_back();
            return p;
        }
        const size_t n = (size_t)1 << cls;
        if (used_ + n > cap_) {
            cap_ = std::max<size_t>(n, (size_t)1 << 22);
            chunks_.emplace_back(new Edge[cap_]);
            used_ = 0;
        }
        Edge* p = chunks_.back().get() + used_;
        used_ += n;
        return p;
    }
    void give_back(Edge* p, int cls) { free_[cls].push_back(p); }

private:
    std::vector<std::unique_ptr<Edge[]>> chunks_;
    size_t used_ = 0, cap_ = 0;
    std::vector<Edge*> free_[40];
};

// Step I.  parent[v] = community v was merged into (-1: root); first_child / next_sibling list
// every community's children from the last merged to the first.
// `work` counts the edge records visited; when it exceeds `work_limit` (> 0) the
// construction stops early and returns false.
bool build_dendrogram(int64_t M, const int64_t* gptr, const int32_t* gadj,
                      std::vector<int32_t>& parent, std::vector<int32_t>& first_child,
                      std::vector<int32_t>& next_sibling, int64_t work_limit, int64_t& work) {
    const int64_t two_m = gptr[M];
    // visiting order: counting sort by degree, stable in the id
    std::vector<int32_t> order(M);
    {
        int64_t maxdeg = 0;
        for (int64_t i = 0; i < M; ++i) maxdeg = std::max(maxdeg, gptr[i + 1] - gptr[i]);
        std::vector<int64_t> start(maxdeg + 2, 0);
        for (int64_t i = 0; i < M; ++i) start[gptr[i + 1] - gptr[i] + 1]++;
        for (int64_t d = 0; d <= maxdeg; ++d) start[d + 1] += start[d];
        for (int64_t i = 0; i < M; ++i) order[start[gptr[i + 1] - gptr[i]]++] = (int32_t)i;
    }
    // What a vertex's own turn reads and writes, in one 24-byte record: consecutive turns visit
    // unrelated ids, so with one array per field every field was a cache miss of its own.
    struct Node {
        int32_t parent = -1;
        int32_t next_sibling = -1;   // next child of the same parent, in reverse merge order
        Edge* agg_ptr = nullptr;     // community edges as of the vertex's turn (kept until the parent's turn)
        int32_t agg_len = 0;
    };
    std::vector<Node> node(M);
    // A merge touches the community joined only through compact arrays (the head of its child
    // list and whether it has had its turn), not through its record: which community that is
    // is known only when the gains are, so nothing can be requested ahead for it.  Children are
    // pushed at the front; their order is immaterial for the sums of Step I, and the caller
    // reads the lists back to front to get the merge order.
    std::vector<int32_t>& head = first_child;
    head.assign(M, -1);
    std::vector<uint8_t> done(M, 0);
    // What every edge record touches stays in compact arrays (they are hit far more often and
    // should stay as cache-resident as they can): union-find links, scratch weights, degree sums.
    std::vector<int32_t> up(M);
    std::vector<int64_t> dsum(M);
    EdgeArena arena;
    std::vector<uint32_t> weight(M, 0);     // scratch: weight towards each community
    std::vector<int32_t> touched;
    for (int64_t i = 0; i < M; ++i) { up[i] = (int32_t)i; dsum[i] = gptr[i + 1] - gptr[i]; }
    auto find = [&](int32_t x) {  // union-find root with full path compression
        int32_t r = x;
        while (up[r] != r) r = up[r];
        while (up[x] != r) { const int32_t nx = up[x]; up[x] = r; x = nx; }
        return r;
    };
    work = 0;
    // Each turn runs in streaming passes over the gathered edge records, so that the cache misses
    // of one pass are all in flight together: (1) collect the records and prefetch their
    // union-find cells, (2) hop once and prefetch the next cell, (3) resolve roots and prefetch
    // their weight cells, (4) accumulate.  The records of the coming turns are requested ahead:
    // record, row pointer and list head kFar turns ahead, then the adjacency row and the first
    // child's record kMid turns ahead, then that child's edge list kNear turns ahead.
    constexpr int64_t kFar = 24, kMid = 16, kNear = 8;
    std::vector<Edge> buf(1024);
    touched.resize(1024);
    for (int64_t step = 0; step < M; ++step) {
        const int32_t v = order[step];
        if (work_limit > 0 && work > work_limit) return false;
        if (step + kFar < M) {
            const int32_t f = order[step + kFar];
            __builtin_prefetch(&node[f]);
            __builtin_prefetch(&gptr[f]);
            __builtin_prefetch(&head[f]);
        }
        if (step + kMid < M) {
            const int32_t n = order[step + kMid];
            __builtin_prefetch(&gadj[gptr[n]]);
            if (head[n] >= 0) __builtin_prefetch(&node[head[n]]);
        }
        if (step + kNear < M) {
            const int32_t c = head[order[step + kNear]];
            if (c >= 0) {
                __builtin_prefetch(node[c].agg_ptr);
                if (node[c].next_sibling >= 0) __builtin_prefetch(&node[node[c].next_sibling]);
            }
        }
        // size the record buffer once per turn (own adjacency + the children's lists), then fill it
        size_t n_rec = (size_t)(gptr[v + 1] - gptr[v]);
        for (int32_t c = head[v]; c >= 0; c = node[c].next_sibling) n_rec += (size_t)node[c].agg_len;
        if (buf.size() < n_rec) buf.resize(std::max(n_rec, buf.size() * 2));
        if (touched.size() < n_rec) touched.resize(std::max(n_rec, touched.size() * 2));
        Edge* out = buf.data();
        for (int64_t p = gptr[v]; p < gptr[v + 1]; ++p) {
            __builtin_prefetch(&up[gadj[p]]);
            *out++ = Edge{gadj[p], 1u};
        }
        for (int32_t c = head[v]; c >= 0; c = node[c].next_sibling) {
            const Edge* list = node[c].agg_ptr;
            const int32_t n = node[c].agg_len;
            const int32_t nc = node[c].next_sibling;
            if (nc >= 0) __builtin_prefetch(&node[nc]);
            for (int32_t k = 0; k < n; ++k) {
                __builtin_prefetch(&up[list[k].to]);
                *out++ = list[k];
            }
            if (list) arena.give_back(node[c].agg_ptr, EdgeArena::size_class((size_t)n));
            node[c].agg_ptr = nullptr;
        }
        Edge* const rec = buf.data();
        work += (int64_t)n_rec + 1;
        for (size_t i = 0; i < n_rec; ++i) {  // one hop up, and ask for the next cell
            rec[i].to = up[rec[i].to];
            __builtin_prefetch(&up[rec[i].to]);
        }
        for (size_t i = 0; i < n_rec; ++i) {
            rec[i].to = find(rec[i].to);
            __builtin_prefetch(&weight[rec[i].to]);
            __builtin_prefetch(&dsum[rec[i].to]);
        }
        int32_t* const tch = touched.data();
        size_t n_touched = 0;
        for (size_t i = 0; i < n_rec; ++i) {
            const int32_t r = rec[i].to;
            if (r == v) continue;
            tch[n_touched] = r;
            n_touched += weight[r] == 0;
            weight[r] += rec[i].w;
        }
        int32_t best = -1;
        int64_t best_s = 0;
        const int64_t dv = dsum[v];
        for (size_t i = 0; i < n_touched; ++i) {
            const int32_t r = tch[i];
            int64_t s = (int64_t)weight[r] * two_m - dsum[r] * dv;
            if (best < 0 || s > best_s || (s == best_s && r < best)) { best = r; best_s = s; }
        }
        const bool merge = best >= 0 && best_s > 0;
        // v's edge list is needed later only if the community it joins has its turn still ahead
        if (merge && !done[best]) {
            Edge* mine = arena.take(EdgeArena::size_class(n_touched));
            for (size_t i = 0; i < n_touched; ++i) mine[i] = Edge{tch[i], weight[tch[i]]};
            node[v].agg_ptr = mine;
            node[v].agg_len = (int32_t)n_touched;
        }
        for (size_t i = 0; i < n_touched; ++i) weight[tch[i]] = 0;
        if (merge) {
            node[v].parent = best;
            up[v] = best;
            node[v].next_sibling = head[best];
            head[best] = v;
            dsum[best] += dsum[v];
        }
        done[v] = 1;
    }
    parent.resize(M);
    next_sibling.resize(M);
    for (int64_t i = 0; i < M; ++i) {
        parent[i] = node[i].parent;
        next_sibling[i] = node[i].next_sibling;
    }
    return true;
}

}  // namespace

namespace {

// leaf sequence: roots by ascending id; a root, then its children's subtrees in merge
// order; each tree's sequence is cut into segments of at most seg_len leaves.  The child lists
// (first_child / next_sibling) run from the last merged child to the first.
void leaf_sequence(int64_t M, const std::vector<int32_t>& parent, const std::vector<int32_t>& first_child,
                   const std::vector<int32_t>& next_sibling, int32_t seg_len, std::vector<int32_t>& seq,
                   std::vector<int64_t>& seg_start) {
    seq.clear();
    seg_start.clear();
    seq.reserve(M);
    std::vector<int32_t> stack;
    for (int64_t r = 0; r < M; ++r) {
        if (parent[r] >= 0) continue;
        const int64_t tree_begin = (int64_t)seq.size();
        // iterative pre-order; the child lists run from the last merged to the first, so pushing
        // them in list order leaves the first merged child on top
        stack.push_back((int32_t)r);
        while (!stack.empty()) {
            int32_t x = stack.back();
            stack.pop_back();
            seq.push_back(x);
            for (int32_t c = first_child[x]; c >= 0; c = next_sibling[c]) stack.push_back(c);
        }
        for (int64_t s = tree_begin; s < (int64_t)seq.size(); s += seg_len) seg_start.push_back(s);
    }
    seg_start.push_back(M);
}

}  // namespace

bool build_dendrogram_host(int64_t M, const int64_t* gptr, const int32_t* gadj, int32_t seg_len, double work_budget,
                           std::vector<int32_t>& parent, std::vector<int32_t>& seq, std::vector<int64_t>& seg_start,
                           double* work_ratio) {
    std::vector<int32_t> first_child, next_sibling;
    const int64_t graph_size = gptr[M] + M;
    int64_t work = 0;
    const bool complete = build_dendrogram(M, gptr, gadj, parent, first_child, next_sibling,
                                           work_budget > 0 ? (int64_t)(work_budget * (double)graph_size) : 0, work);
    if (work_ratio) *work_ratio = graph_size ? (double)work / (double)graph_size : 0.0;
    if (!complete) return false;
    leaf_sequence(M, parent, first_child, next_sibling, seg_len, seq, seg_start);
    return true;
}

void leaf_sequence_from_parents(int64_t M, const std::vector<int32_t>& parent, const std::vector<int32_t>& order,
                                int32_t seg_len, std::vector<int32_t>& seq, std::vector<int64_t>& seg_start) {
    // a vertex is merged at its own turn, so visiting order is merge order: pushing each child at the
    // front of its parent's list leaves the lists running from the last merged child to the first
    std::vector<int32_t> first_child(M, -1), next_sibling(M, -1);
    for (int64_t k = 0; k < M; ++k) {
        const int32_t v = order[k], p = parent[v];
        if (p < 0) continue;
        next_sibling[v] = first_child[p];
        first_child[p] = v;
    }
    leaf_sequence(M, parent, first_child, next_sibling, seg_len, seq, seg_start);
}

}  // namespace accspmm
