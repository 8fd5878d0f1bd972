// Seeded synthetic workload generators (inputs only).
//
// This translation unit produces the sparse matrices (CSR, fp16 values) and dense
// fp16 matrices that both the GPU library's tests and the CPU oracle's tests read.
// It contains no SpMM arithmetic, no tile format and no reordering: only random
// structure and random values.  Every random number is a pure function of
// (seed, stream, counter), so generation is order-independent and thread-parallel.
//
// The shapes follow the kind of inputs the Acc-SpMM paper evaluates on (Table 1:
// square graph adjacency matrices with small and large average row length; Section
// 4.1: feature widths of 128..512): power-law graphs, a regular stencil, a graph with
// hidden communities and a uniform random matrix.
//
// Build: g++ -O3 -fopenmp -shared -fPIC gen.cpp -o libworkloads.so
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <parallel/algorithm>
#include <vector>

namespace {

inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

// Counter-based generator: 64 random bits for (seed, stream, idx).
inline uint64_t rnd(uint64_t seed, uint64_t stream, uint64_t idx) {
    return mix64(mix64(seed + stream * 0xD1342543DE82EF95ULL) ^ idx);
}

inline double u01(uint64_t r) { return (double)(r >> 11) * (1.0 / 9007199254740992.0); }

// float -> IEEE binary16 bits, round-to-nearest-even, with subnormals and overflow to inf.
inline uint16_t f32_to_f16(float f) {
    uint32_t x;
    std::memcpy(&x, &f, 4);
    uint32_t sign = (x >> 16) & 0x8000u;
    uint32_t absx = x & 0x7FFFFFFFu;
    if (absx >= 0x7F800000u) return (uint16_t)(sign | (absx > 0x7F800000u ? 0x7E00u : 0x7C00u));
    if (absx >= 0x477FF000u) return (uint16_t)(sign | 0x7C00u);  // rounds to >= 65520 -> inf
    if (absx < 0x33000001u) return (uint16_t)sign;               // <= 2^-25 -> 0 (tie to even)
    int e = (int)(absx >> 23) - 127;
    uint32_t m = (absx & 0x7FFFFFu) | 0x800000u;
    int shift = (e < -14) ? (13 + (-14 - e)) : 13;  // bits dropped from the 24-bit significand
    uint32_t q = m >> shift;
    uint32_t rem = m & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (q & 1u))) q++;
    uint32_t h;
    if (e < -14) h = q;                                    // subnormal (q may carry into exponent 1)
    else h = ((uint32_t)(e + 15) << 10) + (q - 0x400u);    // q in [0x400,0x800]; carry bumps exponent
    return (uint16_t)(sign | h);
}

enum : uint64_t {
    S_STRUCT = 1,   // structure draws (edges, columns)
    S_VALUE = 2,    // A values, keyed by row*K+col
    S_DENSE = 3,    // B values, keyed by element index
    S_PERM = 4,     // vertex relabelling
    S_RETRY = 16,   // + attempt number for rejection loops
};

struct Csr {
    int64_t M = 0, K = 0, nnz = 0;
    std::vector<int32_t> rowptr, colidx;
    std::vector<uint16_t> vals;
};

inline uint16_t value_u(uint64_t seed, int64_t K, int64_t i, int64_t j, float lo, float hi) {
    double u = u01(rnd(seed, S_VALUE, (uint64_t)i * (uint64_t)K + (uint64_t)j));
    return f32_to_f16((float)(lo + (hi - lo) * u));
}

// keys are (row << 32 | col), sorted, with UINT64_MAX entries (dropped samples) at the end.
Csr* csr_from_sorted_keys(std::vector<uint64_t>& keys, int64_t M, int64_t K, uint64_t seed, float lo, float hi) {
    Csr* out = new Csr;
    out->M = M;
    out->K = K;
    size_t n = keys.size();
    // de-duplicate in place
    size_t w = 0;
    for (size_t r = 0; r < n; ++r) {
        if (keys[r] == UINT64_MAX) break;
        if (w == 0 || keys[r] != keys[w - 1]) keys[w++] = keys[r];
    }
    out->nnz = (int64_t)w;
    out->rowptr.assign(M + 1, 0);
    out->colidx.resize(w);
    out->vals.resize(w);
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < (int64_t)w; ++p) {
        int64_t i = (int64_t)(keys[p] >> 32), j = (int64_t)(keys[p] & 0xFFFFFFFFu);
        out->colidx[p] = (int32_t)j;
        out->vals[p] = value_u(seed, K, i, j, lo, hi);
    }
    for (size_t p = 0; p < w; ++p) out->rowptr[(keys[p] >> 32) + 1]++;
    for (int64_t i = 0; i < M; ++i) out->rowptr[i + 1] += out->rowptr[i];
    return out;
}

}  // namespace

extern "C" {

int64_t wl_csr_nnz(const void* h) { return ((const Csr*)h)->nnz; }
int64_t wl_csr_rows(const void* h) { return ((const Csr*)h)->M; }
void wl_csr_copy(const void* h, int32_t* rowptr, int32_t* colidx, uint16_t* vals) {
    const Csr* c = (const Csr*)h;
    std::memcpy(rowptr, c->rowptr.data(), sizeof(int32_t) * (c->M + 1));
    if (c->nnz) {
        std::memcpy(colidx, c->colidx.data(), sizeof(int32_t) * c->nnz);
        std::memcpy(vals, c->vals.data(), sizeof(uint16_t) * c->nnz);
    }
}
void wl_csr_free(void* h) { delete (Csr*)h; }

uint16_t wl_f32_to_f16(float f) { return f32_to_f16(f); }
uint64_t wl_rnd(uint64_t seed, uint64_t stream, uint64_t idx) { return rnd(seed, stream, idx); }

// Uniform random rows: every row has exactly `per_row` distinct columns drawn uniformly
// from [0,K); values U[lo,hi].
void* wl_uniform(int64_t M, int64_t K, int32_t per_row, uint64_t seed, float lo, float hi) {
    if (per_row > K) return nullptr;
    Csr* out = new Csr;
    out->M = M;
    out->K = K;
    out->nnz = M * per_row;
    out->rowptr.resize(M + 1);
    out->colidx.resize(out->nnz);
    out->vals.resize(out->nnz);
    for (int64_t i = 0; i <= M; ++i) out->rowptr[i] = (int32_t)(i * per_row);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        int32_t* c = out->colidx.data() + i * per_row;
        for (int s = 0; s < per_row; ++s) {
            for (uint64_t attempt = 0;; ++attempt) {
                int32_t cand = (int32_t)(rnd(seed, S_STRUCT + S_RETRY * attempt, (uint64_t)(i * per_row + s)) % (uint64_t)K);
                bool dup = false;
                for (int t = 0; t < s; ++t) dup |= (c[t] == cand);
                if (!dup) { c[s] = cand; break; }
            }
        }
        std::sort(c, c + per_row);
        for (int s = 0; s < per_row; ++s) out->vals[i * per_row + s] = value_u(seed, K, i, c[s], lo, hi);
    }
    return out;
}

// R-MAT graph with 2^scale vertices.  Each of n_samples edges picks one quadrant per
// level with probabilities (a, b, c, 1-a-b-c) quantised to 1/65536.  Duplicates are
// removed.  If symmetrize != 0, self loops are dropped and (j,i) is added for every (i,j).
void* wl_rmat(int32_t scale, int64_t n_samples, double a, double b, double c, uint64_t seed,
              int32_t symmetrize, float lo, float hi) {
    int64_t V = (int64_t)1 << scale;
    uint32_t ta = (uint32_t)std::lround(a * 65536.0);
    uint32_t tb = ta + (uint32_t)std::lround(b * 65536.0);
    uint32_t tc = tb + (uint32_t)std::lround(c * 65536.0);
    std::vector<uint64_t> keys((size_t)n_samples * (symmetrize ? 2 : 1));
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < n_samples; ++e) {
        uint64_t i = 0, j = 0, bits = 0;
        for (int l = 0; l < scale; ++l) {
            if ((l & 3) == 0) bits = rnd(seed, S_STRUCT + S_RETRY * (uint64_t)(l >> 2), (uint64_t)e);
            uint32_t u = (uint32_t)(bits & 0xFFFFu);
            bits >>= 16;
            uint64_t bi = (u >= tb), bj = (u >= ta && u < tb) || (u >= tc);
            i = (i << 1) | bi;
            j = (j << 1) | bj;
        }
        if (symmetrize) {
            if (i == j) {
                keys[2 * e] = keys[2 * e + 1] = UINT64_MAX;
            } else {
                keys[2 * e] = (i << 32) | j;
                keys[2 * e + 1] = (j << 32) | i;
            }
        } else {
            keys[e] = (i << 32) | j;
        }
    }
    __gnu_parallel::sort(keys.begin(), keys.end());
    return csr_from_sorted_keys(keys, V, V, seed, lo, hi);
}

// 27-point stencil on an n*n*n grid, natural lexicographic order (x fastest), no
// wrap-around.  Diagonal entries hold `diag`; the others are U[lo,hi].
void* wl_stencil27(int32_t n, uint64_t seed, float diag, float lo, float hi) {
    int64_t M = (int64_t)n * n * n;
    Csr* out = new Csr;
    out->M = M;
    out->K = M;
    out->rowptr.resize(M + 1);
    auto span = [n](int v) { return (v > 0) + 1 + (v < n - 1); };
    out->rowptr[0] = 0;
    for (int64_t r = 0; r < M; ++r) {
        int x = (int)(r % n), y = (int)((r / n) % n), z = (int)(r / ((int64_t)n * n));
        out->rowptr[r + 1] = out->rowptr[r] + span(x) * span(y) * span(z);
    }
    out->nnz = out->rowptr[M];
    out->colidx.resize(out->nnz);
    out->vals.resize(out->nnz);
    uint16_t dh = f32_to_f16(diag);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; ++r) {
        int x = (int)(r % n), y = (int)((r / n) % n), z = (int)(r / ((int64_t)n * n));
        int64_t p = out->rowptr[r];
        for (int dz = -1; dz <= 1; ++dz)
            for (int dy = -1; dy <= 1; ++dy)
                for (int dx = -1; dx <= 1; ++dx) {
                    int xx = x + dx, yy = y + dy, zz = z + dz;
                    if (xx < 0 || yy < 0 || zz < 0 || xx >= n || yy >= n || zz >= n) continue;
                    int64_t col = xx + (int64_t)n * (yy + (int64_t)n * zz);
                    out->colidx[p] = (int32_t)col;
                    out->vals[p] = (col == r) ? dh : value_u(seed, M, r, col, lo, hi);
                    ++p;
                }
    }
    return out;
}

// Stochastic block model with hidden communities: V vertices in consecutive communities
// of `csize`; each intra-community pair is an edge with probability p_in; V*inter_deg/2
// further pairs with endpoints in different communities are drawn uniformly.  The graph
// is symmetric without self loops.  If relabel != 0 the vertex ids are then permuted by a
// seeded random permutation (rows and columns alike), which hides the blocks.
void* wl_sbm(int64_t V, int32_t csize, double p_in, double inter_deg, uint64_t seed, int32_t relabel,
             float lo, float hi) {
    int64_t ncomm = V / csize;
    int64_t pairs_per = (int64_t)csize * (csize - 1) / 2;
    int64_t n_inter = (int64_t)std::llround((double)V * inter_deg / 2.0);
    std::vector<int64_t> label(V);
    if (relabel) {
        std::vector<uint64_t> pk(V);
        for (int64_t v = 0; v < V; ++v) pk[v] = (rnd(seed, S_PERM, (uint64_t)v) & ~0xFFFFFFFFULL) | (uint64_t)v;
        std::sort(pk.begin(), pk.end());
        for (int64_t r = 0; r < V; ++r) label[pk[r] & 0xFFFFFFFFu] = r;
    } else {
        for (int64_t v = 0; v < V; ++v) label[v] = v;
    }
    std::vector<uint64_t> keys((size_t)2 * (ncomm * pairs_per + n_inter), UINT64_MAX);
    uint64_t thr = (uint64_t)(p_in * 9007199254740992.0);
#pragma omp parallel for schedule(static)
    for (int64_t cc = 0; cc < ncomm; ++cc) {
        int64_t q = 0;
        for (int x = 0; x < csize; ++x)
            for (int y = x + 1; y < csize; ++y, ++q) {
                uint64_t idx = (uint64_t)(cc * pairs_per + q);
                if ((rnd(seed, S_STRUCT, idx) >> 11) < thr) {
                    uint64_t i = (uint64_t)label[cc * csize + x], j = (uint64_t)label[cc * csize + y];
                    keys[2 * idx] = (i << 32) | j;
                    keys[2 * idx + 1] = (j << 32) | i;
                }
            }
    }
    int64_t base = ncomm * pairs_per;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < n_inter; ++e) {
        for (uint64_t attempt = 0;; ++attempt) {
            uint64_t r = rnd(seed, S_STRUCT + S_RETRY * (attempt + 1), (uint64_t)e);
            int64_t x = (int64_t)((r >> 32) % (uint64_t)V), y = (int64_t)((r & 0xFFFFFFFFu) % (uint64_t)V);
            if (x / csize == y / csize) continue;
            uint64_t i = (uint64_t)label[x], j = (uint64_t)label[y];
            keys[2 * (base + e)] = (i << 32) | j;
            keys[2 * (base + e) + 1] = (j << 32) | i;
            break;
        }
    }
    __gnu_parallel::sort(keys.begin(), keys.end());
    return csr_from_sorted_keys(keys, V, V, seed, lo, hi);
}

// Dense row-major fp16 matrix, rows*cols elements.  kind 0: U[p0,p1]; kind 1: normal with
// mean p0 and standard deviation p1 (Box-Muller, one pair of outputs per pair of elements).
void wl_dense(int64_t rows, int64_t cols, uint64_t seed, int32_t kind, float p0, float p1, uint16_t* out) {
    int64_t n = rows * cols;
    if (kind == 0) {
#pragma omp parallel for schedule(static)
        for (int64_t e = 0; e < n; ++e) out[e] = f32_to_f16((float)(p0 + (p1 - p0) * u01(rnd(seed, S_DENSE, (uint64_t)e))));
    } else {
        int64_t np = (n + 1) / 2;
#pragma omp parallel for schedule(static)
        for (int64_t p = 0; p < np; ++p) {
            double u1 = ((double)(rnd(seed, S_DENSE, (uint64_t)(2 * p)) >> 11) + 1.0) * (1.0 / 9007199254740992.0);
            double u2 = u01(rnd(seed, S_DENSE, (uint64_t)(2 * p + 1)));
            double rad = std::sqrt(-2.0 * std::log(u1)), ang = 6.283185307179586476925 * u2;
            out[2 * p] = f32_to_f16((float)(p0 + p1 * rad * std::cos(ang)));
            if (2 * p + 1 < n) out[2 * p + 1] = f32_to_f16((float)(p0 + p1 * rad * std::sin(ang)));
        }
    }
}

}  // extern "C"
