// CPU oracle for the Acc-SpMM hot path.  TEST INFRASTRUCTURE ONLY.
//
// Plain, slow, fp64/integer reference implementations of what the GPU library computes.
// Only tests, the smoke check and the benchmark's cpu_baseline leg may call this; the
// product path never does, and this file shares no code with the GPU library.
//
//   orc_spmm*        C = A.B from the definition of SpMM (paper, Section 5 first
//                    sentence; CSR as in Section 2.2), in fp64, plus sum |a||b|.
//   orc_encode/decode  the bitmap tile format of Section 3.3 (RowWindowOffset, TCOffset,
//                    SparseAToB, TCLocalBit, packed values; decode by popcount of lower
//                    bits), generalised from 8x8 tiles to WH x TW tiles.
//   orc_dendrogram / orc_ordering / orc_reorder
//                    the two steps of Algorithm 1 (Section 3.2).
//   orc_ibd          the imbalance degree of Eq. 3 (Section 3.5).
//
// Readings of points the paper leaves open are listed next to each function.
//
// Parity status: orc_spmm, orc_encode, orc_decode and orc_ibd are pinned by tests that do
// not depend on this file (dense brute force, identity/permutation matrices, hand-worked
// tiles, the closed-form size of Section 3.3, direct numpy evaluation).
// orc_dendrogram / orc_ordering: PARITY UNPINNED against the paper (its worked example
// lives in a figure that is not available); they are pinned against a literal pure-Python
// transcription of the same steps and hand-worked small graphs.
//
// Build: g++ -O2 -fopenmp -shared -fPIC oracle.cpp -o liboracle.so
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <map>
#include <utility>
#include <vector>

namespace {

// number of set bits of a tile's bitmap strictly below bit index `bit`
inline int rank_below(const uint64_t* words, int bit) {
    int rank = 0;
    for (int k = 0; k < bit / 64; ++k) rank += __builtin_popcountll(words[k]);
    if (bit % 64) rank += __builtin_popcountll(words[bit / 64] & (((uint64_t)1 << (bit % 64)) - 1));
    return rank;
}

// IEEE binary16 bit pattern -> double (exact).
inline double h2d(uint16_t h) {
    int s = h >> 15, e = (h >> 10) & 31, f = h & 1023;
    double v;
    if (e == 0) v = std::ldexp((double)f, -24);
    else if (e == 31) v = f ? NAN : INFINITY;
    else v = std::ldexp((double)(f + 1024), e - 25);
    return s ? -v : v;
}

// bfloat16 bit pattern -> double (exact): sign, 8 exponent bits (bias 127), 7 fraction bits,
// i.e. the upper half of an IEEE binary32.
inline double bf2d(uint16_t h) {
    int s = h >> 15, e = (h >> 7) & 255, f = h & 127;
    double v;
    if (e == 0) v = std::ldexp((double)f, -133);            // subnormal: f * 2^-7 * 2^-126
    else if (e == 255) v = f ? NAN : INFINITY;
    else v = std::ldexp((double)(f + 128), e - 134);        // (1 + f/128) * 2^(e-127)
    return s ? -v : v;
}

// value_type: 0 = IEEE binary16, 1 = bfloat16
inline double widen(uint16_t h, int value_type) { return value_type == 1 ? bf2d(h) : h2d(h); }

}  // namespace

// Long runs (the full-size reordering takes minutes) can report how far they are: a line on
// stderr every g_progress_every steps of Step I.  0 (default) prints nothing.  No effect on
// any result.
static int64_t g_progress_every = 0;

extern "C" {

void orc_set_progress(int64_t every) { g_progress_every = every > 0 ? every : 0; }

double orc_f16_to_f64(uint16_t h) { return h2d(h); }
double orc_bf16_to_f64(uint16_t h) { return bf2d(h); }

// C[i][j] = sum_p A.val[p] * B[A.col[p]][j] over the stored entries p of row i, in fp64
// (definition of SpMM).  bound[i][j] = sum_p |A.val[p]| * |B[A.col[p]][j]| (may be null).
// `rows` selects which rows to compute (null = rows 0..nrows-1); output row r of C/bound
// corresponds to rows[r].
// `value_type` names the 16-bit type of vals and B (0 = binary16, the type of the benchmark
// workloads; 1 = bfloat16).
void orc_spmm_rows_typed(int64_t nrows, const int64_t* rows, int64_t N, const int32_t* rowptr,
                         const int32_t* colidx, const uint16_t* vals, const uint16_t* B, double* C,
                         double* bound, int value_type) {
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t i = rows ? rows[r] : r;
        double* c = C + r * N;
        double* bd = bound ? bound + r * N : nullptr;
        for (int64_t j = 0; j < N; ++j) c[j] = 0.0;
        if (bd) for (int64_t j = 0; j < N; ++j) bd[j] = 0.0;
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            double a = widen(vals[p], value_type);
            const uint16_t* brow = B + (int64_t)colidx[p] * N;
            for (int64_t j = 0; j < N; ++j) {
                double b = widen(brow[j], value_type);
                c[j] += a * b;
                if (bd) bd[j] += std::fabs(a) * std::fabs(b);
            }
        }
    }
}

void orc_spmm_rows(int64_t nrows, const int64_t* rows, int64_t N, const int32_t* rowptr,
                   const int32_t* colidx, const uint16_t* vals, const uint16_t* B, double* C,
                   double* bound) {
    orc_spmm_rows_typed(nrows, rows, N, rowptr, colidx, vals, B, C, bound, 0);
}

// Sampled dense-dense product: for every stored entry p = (i, j) of the pattern,
// out[p] = scale_p * sum_f X[i][f] * Y[j][f] in fp64, with scale_p = the entry's value if
// `vals` is given, else 1; bound[p] = |scale_p| * sum_f |X[i][f]| * |Y[j][f]| (may be null).
// X is M x N, Y is K x N, both row-major bit patterns of `value_type`.  (Not an operation of
// the paper; the definition is the standard one of the SpMM / SDDMM pair of GNN layers.)
void orc_sddmm(int64_t M, int64_t N, const int32_t* rowptr, const int32_t* colidx, const uint16_t* vals,
               const uint16_t* X, const uint16_t* Y, double* out, double* bound, int value_type) {
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = 0; i < M; ++i) {
        const uint16_t* x = X + i * N;
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            const uint16_t* y = Y + (int64_t)colidx[p] * N;
            double dot = 0.0, mag = 0.0;
            for (int64_t f = 0; f < N; ++f) {
                const double a = widen(x[f], value_type), b = widen(y[f], value_type);
                dot += a * b;
                mag += std::fabs(a) * std::fabs(b);
            }
            const double scale = vals ? widen(vals[p], value_type) : 1.0;
            out[p] = scale * dot;
            if (bound) bound[p] = std::fabs(scale) * mag;
        }
    }
}

void orc_spmm(int64_t M, int64_t N, const int32_t* rowptr, const int32_t* colidx, const uint16_t* vals,
              const uint16_t* B, double* C, double* bound) {
    orc_spmm_rows(M, nullptr, N, rowptr, colidx, vals, B, C, bound);
}

// ---------------------------------------------------------------------------------------
// Tile format (Section 3.3), WH rows per row window, TW condensed columns per tile.
//
// Reordered row r is input row perm[r] (perm == null: identity).  Window w holds reordered
// rows [w*WH, min((w+1)*WH, M)).  Readings: condensed columns of a window are its distinct
// column indices in ascending order; bit index of local position (r,c) is r*TW + c, bit b
// of the tile lives in word b/64 at bit b%64 (LSB first); the unused SparseAToB slots of a
// window's last tile repeat the window's last column; values of a tile are packed in
// ascending bit order (so that "popcount of the lower bits" is the value's offset).
//
// Call with the output pointers null to get the tile count T; then call again with
//   row_window_offset[W+1], tc_offset[T+1], sparse_a_to_b[T*TW], tc_local_bit[T*NW]
//   (NW = ceil(WH*TW/64)), packed_vals[nnz].
// Returns T, or -1 on a duplicate column inside a row.
int64_t orc_encode(int64_t M, const int32_t* rowptr, const int32_t* colidx, const uint16_t* vals,
                   const int32_t* perm, int32_t WH, int32_t TW, int32_t* row_window_offset,
                   int32_t* tc_offset, int32_t* sparse_a_to_b, uint64_t* tc_local_bit,
                   uint16_t* packed_vals) {
    const int64_t W = (M + WH - 1) / WH;
    const int NW = (WH * TW + 63) / 64;
    const bool fill = row_window_offset != nullptr;
    int64_t T = 0;
    if (fill) { row_window_offset[0] = 0; tc_offset[0] = 0; }
    std::vector<int32_t> cols;
    for (int64_t w = 0; w < W; ++w) {
        const int64_t r0 = w * WH, r1 = std::min<int64_t>(M, r0 + WH);
        cols.clear();
        for (int64_t r = r0; r < r1; ++r) {
            int64_t i = perm ? perm[r] : r;
            for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) cols.push_back(colidx[p]);
        }
        std::sort(cols.begin(), cols.end());
        cols.erase(std::unique(cols.begin(), cols.end()), cols.end());
        const int64_t d = (int64_t)cols.size();
        const int64_t Tw = (d + TW - 1) / TW;
        if (fill) {
            for (int64_t t = 0; t < Tw; ++t) {
                const int64_t g = T + t;
                for (int c = 0; c < TW; ++c)
                    sparse_a_to_b[g * TW + c] = cols[std::min<int64_t>(t * TW + c, d - 1)];
                for (int k = 0; k < NW; ++k) tc_local_bit[g * NW + k] = 0;
            }
            // set bits
            for (int64_t r = r0; r < r1; ++r) {
                int64_t i = perm ? perm[r] : r;
                for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
                    int64_t cc = std::lower_bound(cols.begin(), cols.end(), colidx[p]) - cols.begin();
                    int64_t g = T + cc / TW;
                    int bit = (int)((r - r0) * TW + cc % TW);
                    uint64_t& word = tc_local_bit[g * NW + bit / 64];
                    if (word >> (bit % 64) & 1) return -1;
                    word |= (uint64_t)1 << (bit % 64);
                }
            }
            // offsets
            for (int64_t t = 0; t < Tw; ++t) {
                int cnt = 0;
                for (int k = 0; k < NW; ++k) cnt += __builtin_popcountll(tc_local_bit[(T + t) * NW + k]);
                tc_offset[T + t + 1] = tc_offset[T + t] + cnt;
            }
            // values: rank of a bit = number of set bits below it inside the tile
            for (int64_t r = r0; r < r1; ++r) {
                int64_t i = perm ? perm[r] : r;
                for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
                    int64_t cc = std::lower_bound(cols.begin(), cols.end(), colidx[p]) - cols.begin();
                    int64_t g = T + cc / TW;
                    int bit = (int)((r - r0) * TW + cc % TW);
                    packed_vals[tc_offset[g] + rank_below(tc_local_bit + g * NW, bit)] = vals[p];
                }
            }
            row_window_offset[w + 1] = (int32_t)(T + Tw);
        }
        T += Tw;
    }
    return T;
}

// Inverse of orc_encode: rebuilds the reordered matrix as CSR (out_rowptr[M+1],
// out_colidx[nnz], out_vals[nnz]; row r of the output is reordered row r, columns
// ascending).  A position holds vals[tc_offset[g] + popcount(lower bits)] if its bit is
// set (Section 3.3, decompression), otherwise it is a structural zero and is not emitted.
void orc_decode(int64_t M, int32_t WH, int32_t TW, const int32_t* row_window_offset,
                const int32_t* tc_offset, const int32_t* sparse_a_to_b, const uint64_t* tc_local_bit,
                const uint16_t* packed_vals, int32_t* out_rowptr, int32_t* out_colidx, uint16_t* out_vals) {
    const int64_t W = (M + WH - 1) / WH;
    const int NW = (WH * TW + 63) / 64;
    int64_t q = 0;
    out_rowptr[0] = 0;
    for (int64_t w = 0; w < W; ++w) {
        for (int rl = 0; rl < WH; ++rl) {
            int64_t r = w * WH + rl;
            if (r >= M) break;
            for (int64_t g = row_window_offset[w]; g < row_window_offset[w + 1]; ++g) {
                for (int c = 0; c < TW; ++c) {
                    int bit = rl * TW + c;
                    if (!(tc_local_bit[g * NW + bit / 64] >> (bit % 64) & 1)) continue;
                    out_colidx[q] = sparse_a_to_b[g * TW + c];
                    out_vals[q] = packed_vals[tc_offset[g] + rank_below(tc_local_bit + g * NW, bit)];
                    ++q;
                }
            }
            out_rowptr[r + 1] = (int32_t)q;
        }
    }
}

// ---------------------------------------------------------------------------------------
// Algorithm 1, Step I (dendrogram construction).
//
// Graph: vertex per row/column index (square matrices); undirected unit-weight edge {i,j},
// i != j, iff A_ij or A_ji is stored.  Vertices are visited in ascending degree (ties:
// lower id).  At its turn, v (with everything merged into it so far) is merged into the
// neighbouring community u that maximises the modularity gain, if that gain is positive.
// Reading of Eq. 1: the gain of joining communities u and v is
//   2*( w_uv/(2m) - d_u*d_v/(2m)^2 ),  compared exactly through
//   s(u) = w_uv*2m - d_u*d_v  (ties: lower community id, which is the id of its root).
// Output: parent[v] (-1 for roots), and child_order[v] = the rank of v among the children
// of parent[v] in merge order (0,1,2,...; 0 for roots).
void orc_dendrogram(int64_t M, const int32_t* rowptr, const int32_t* colidx, int32_t* parent,
                    int32_t* child_order) {
    std::vector<std::vector<int32_t>> adj(M);
    for (int64_t i = 0; i < M; ++i)
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            int32_t j = colidx[p];
            if (j == i) continue;
            adj[i].push_back(j);
            adj[j].push_back((int32_t)i);
        }
    int64_t two_m = 0;
    for (int64_t i = 0; i < M; ++i) {
        std::sort(adj[i].begin(), adj[i].end());
        adj[i].erase(std::unique(adj[i].begin(), adj[i].end()), adj[i].end());
        two_m += (int64_t)adj[i].size();
    }
    std::vector<int32_t> order(M);
    for (int64_t i = 0; i < M; ++i) order[i] = (int32_t)i;
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return adj[a].size() < adj[b].size(); });
    std::vector<int64_t> dsum(M);
    std::vector<int32_t> nchild(M, 0);
    // agg[v]: after v's turn, the (community -> weight) edges of v's community at that time
    std::vector<std::vector<std::pair<int32_t, int64_t>>> agg(M);
    std::vector<std::vector<int32_t>> children(M);
    for (int64_t i = 0; i < M; ++i) { parent[i] = -1; child_order[i] = 0; dsum[i] = (int64_t)adj[i].size(); }
    // union-find view of `parent` with path halving (parent itself keeps the merge tree)
    std::vector<int32_t> up(M);
    for (int64_t i = 0; i < M; ++i) up[i] = (int32_t)i;
    auto root = [&](int32_t x) { while (up[x] != x) { up[x] = up[up[x]]; x = up[x]; } return x; };
    for (int64_t t = 0; t < M; ++t) {
        int32_t v = order[t];
        if (g_progress_every && t % g_progress_every == 0) {
            std::fprintf(stderr, "[oracle] dendrogram: vertex %lld of %lld\n", (long long)t, (long long)M);
            std::fflush(stderr);
        }
        std::map<int32_t, int64_t> w;
        for (int32_t y : adj[v]) { int32_t ry = root(y); if (ry != v) w[ry] += 1; }
        for (int32_t c : children[v])
            for (auto& e : agg[c]) { int32_t ry = root(e.first); if (ry != v) w[ry] += e.second; }
        int32_t best = -1;
        int64_t best_s = 0;
        for (auto& e : w) {  // ascending community id: the first maximum wins ties
            int64_t s = e.second * two_m - dsum[e.first] * dsum[v];
            if (best < 0 || s > best_s) { best = e.first; best_s = s; }
        }
        agg[v].assign(w.begin(), w.end());
        for (int32_t c : children[v]) { agg[c].clear(); agg[c].shrink_to_fit(); }
        if (best >= 0 && best_s > 0) {
            parent[v] = best;
            up[v] = best;
            child_order[v] = nchild[best]++;
            children[best].push_back(v);
            dsum[best] += dsum[v];
        }
    }
}

// Algorithm 1, Step II (ordering generation).
//
// Leaf sequence: roots in ascending id; a tree rooted at r lists r first, then the subtree
// of each child in merge order.  Each tree's sequence is cut into consecutive segments of
// at most seg_len leaves.  Inside a segment: take the first unvisited leaf v, give it the
// next new id; then repeatedly pick, among the segment's unvisited leaves, the one whose
// row shares the most column indices with row v (at least one; ties: earliest in the
// sequence), give it the next id and continue from it; when no leaf shares a column the
// chain ends and the scan resumes.  perm[new] = old, iperm[old] = new.
// Reading: the search scope "all leaf nodes" is limited to the segment (the unrestricted
// search is quadratic and contradicts the stated O(n log n)).
void orc_ordering(int64_t M, const int32_t* rowptr, const int32_t* colidx, const int32_t* parent,
                  const int32_t* child_order, int32_t seg_len, int32_t* perm, int32_t* iperm,
                  int32_t* leaf_seq /* may be null: DFS sequence, M entries */,
                  int32_t* seg_start /* may be null: M+1 entries max, terminated by M */) {
    std::vector<std::vector<int32_t>> children(M);
    for (int64_t v = 0; v < M; ++v) if (parent[v] >= 0) {
        auto& ch = children[parent[v]];
        if ((int64_t)ch.size() <= child_order[v]) ch.resize(child_order[v] + 1);
        ch[child_order[v]] = (int32_t)v;
    }
    std::vector<int32_t> seq;
    std::vector<int64_t> starts;  // segment starts
    seq.reserve(M);
    std::vector<std::pair<int32_t, size_t>> stack;
    for (int64_t r = 0; r < M; ++r) {
        if (parent[r] >= 0) continue;
        size_t tree_begin = seq.size();
        stack.push_back({(int32_t)r, 0});
        seq.push_back((int32_t)r);
        while (!stack.empty()) {
            auto& top = stack.back();
            if (top.second < children[top.first].size()) {
                int32_t c = children[top.first][top.second++];
                seq.push_back(c);
                stack.push_back({c, 0});
            } else stack.pop_back();
        }
        for (size_t s = tree_begin; s < seq.size(); s += seg_len) starts.push_back((int64_t)s);
    }
    starts.push_back(M);
    if (leaf_seq) std::copy(seq.begin(), seq.end(), leaf_seq);
    if (seg_start) for (size_t i = 0; i < starts.size(); ++i) seg_start[i] = (int32_t)starts[i];

    const int64_t nseg = (int64_t)starts.size() - 1;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t sgi = 0; sgi < nseg; ++sgi) {
        const int64_t b = starts[sgi], e = starts[sgi + 1], n = e - b;
        // inverted index of the segment: column -> positions (ascending) of rows holding it
        std::vector<std::pair<int32_t, int32_t>> cp;
        for (int64_t q = 0; q < n; ++q) {
            int32_t row = seq[b + q];
            for (int64_t p = rowptr[row]; p < rowptr[row + 1]; ++p) cp.push_back({colidx[p], (int32_t)q});
        }
        std::sort(cp.begin(), cp.end());
        std::vector<char> visited(n, 0);
        std::vector<int32_t> count(n, 0);
        int64_t next = b;
        for (int64_t cur = 0; cur < n; ++cur) {
            if (visited[cur]) continue;
            int64_t v = cur;
            for (;;) {
                visited[v] = 1;
                perm[next++] = seq[b + v];
                std::fill(count.begin(), count.end(), 0);
                int32_t row = seq[b + v];
                for (int64_t p = rowptr[row]; p < rowptr[row + 1]; ++p) {
                    auto lo = std::lower_bound(cp.begin(), cp.end(), std::make_pair(colidx[p], (int32_t)-1));
                    for (; lo != cp.end() && lo->first == colidx[p]; ++lo) count[lo->second]++;
                }
                int64_t best = -1;
                for (int64_t q = 0; q < n; ++q)
                    if (!visited[q] && count[q] >= 1 && (best < 0 || count[q] > count[best])) best = q;
                if (best < 0) break;
                v = best;
            }
        }
    }
    for (int64_t r = 0; r < M; ++r) iperm[perm[r]] = (int32_t)r;
}

void orc_reorder(int64_t M, const int32_t* rowptr, const int32_t* colidx, int32_t seg_len, int32_t* perm,
                 int32_t* iperm) {
    std::vector<int32_t> parent(M), child_order(M);
    orc_dendrogram(M, rowptr, colidx, parent.data(), child_order.data());
    orc_ordering(M, rowptr, colidx, parent.data(), child_order.data(), seg_len, perm, iperm, nullptr, nullptr);
}

// Eq. 3: mean absolute deviation of the number of tiles per row window.
double orc_ibd(int64_t W, const int32_t* row_window_offset) {
    if (W <= 0) return 0.0;
    double avg = (double)(row_window_offset[W] - row_window_offset[0]) / (double)W, s = 0.0;
    for (int64_t w = 0; w < W; ++w) s += std::fabs((double)(row_window_offset[w + 1] - row_window_offset[w]) - avg);
    return s / (double)W;
}

}  // extern "C"
