// Matrix Market coordinate files -> host CSR with 16-bit values, so that the matrices the
// paper evaluates on (SuiteSparse, graph collections; Section 4.1), which ship in this format,
// can be handed to acc_spmm_plan when a user has them.  Host code only.
//
// Supported: "matrix coordinate" with field real / integer / pattern and symmetry general /
// symmetric / skew-symmetric.  Symmetric files store one triangle; the other is mirrored
// (negated for skew-symmetric).  Pattern entries get the value 1.  Entries given more than
// once are summed.  Complex / hermitian and the dense "array" layout are refused.
#include <algorithm>
#include <cctype>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "internal.h"

namespace accspmm {

struct MtxFile {
    int64_t M = 0, K = 0;
    std::vector<int32_t> rowptr, colidx;
    std::vector<uint16_t> vals;
};

namespace {

// float -> IEEE binary16 bits, round to nearest even; overflow gives infinity
uint16_t to_half_bits(float x) {
    uint32_t u;
    std::memcpy(&u, &x, 4);
    const uint32_t sign = (u >> 16) & 0x8000u;
    const uint32_t mag = u & 0x7fffffffu;
    if (mag >= 0x7f800000u) return (uint16_t)(sign | 0x7c00u | ((mag > 0x7f800000u) ? 0x200u : 0u));  // inf / nan
    if (mag >= 0x477ff000u) return (uint16_t)(sign | 0x7c00u);  // rounds to 65536 or more
    if (mag < 0x33000001u) return (uint16_t)sign;               // at most half the smallest subnormal
    int32_t e = (int32_t)(mag >> 23) - 127;
    uint32_t m = (mag & 0x7fffffu) | 0x800000u;                 // 24-bit significand
    int shift = (e < -14) ? (13 + (-14 - e)) : 13;              // bits dropped (subnormal halves drop more)
    uint32_t kept = m >> shift;
    const uint32_t rest = m & ((1u << shift) - 1u), half = 1u << (shift - 1);
    if (rest > half || (rest == half && (kept & 1u))) ++kept;
    if (e < -14) return (uint16_t)(sign | kept);                // subnormal (a carry lands on the smallest normal)
    return (uint16_t)(sign | (((uint32_t)(e + 15) << 10) + (kept - 0x400u)));  // a carry bumps the exponent
}

// float -> bfloat16 bits, round to nearest even
uint16_t to_bf16_bits(float x) {
    uint32_t u;
    std::memcpy(&u, &x, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // nan stays nan
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

std::string lower(std::string s) {
    for (auto& ch : s) ch = (char)std::tolower((unsigned char)ch);
    return s;
}

struct Entry {
    int32_t r, c;
    double v;
};

}  // namespace

MtxFile* read_matrix_market(const char* path, int32_t value_type) {
    if (!path) fail(ACC_SPMM_ERR_INVALID_ARG, "null path");
    if (value_type != ACC_SPMM_FP16 && value_type != ACC_SPMM_BF16)
        fail(ACC_SPMM_ERR_INVALID_ARG, "value_type must be ACC_SPMM_FP16 or ACC_SPMM_BF16");
    std::FILE* f = std::fopen(path, "rb");
    if (!f) fail(ACC_SPMM_ERR_INVALID_ARG, std::string("cannot open ") + path);
    struct Closer {
        std::FILE* f;
        ~Closer() { std::fclose(f); }
    } closer{f};

    std::vector<char> line(1 << 16);
    if (!std::fgets(line.data(), (int)line.size(), f)) fail(ACC_SPMM_ERR_INVALID_ARG, "empty file");
    char banner[64], object[64], layout[64], field[64], symmetry[64];
    if (std::sscanf(line.data(), "%63s %63s %63s %63s %63s", banner, object, layout, field, symmetry) != 5 ||
        lower(banner) != "%%matrixmarket" || lower(object) != "matrix")
        fail(ACC_SPMM_ERR_INVALID_ARG, "not a Matrix Market matrix file (bad header line)");
    if (lower(layout) != "coordinate") fail(ACC_SPMM_ERR_UNSUPPORTED, "only the coordinate layout is supported");
    const std::string fld = lower(field), sym = lower(symmetry);
    const bool pattern = fld == "pattern";
    if (!pattern && fld != "real" && fld != "integer" && fld != "double")
        fail(ACC_SPMM_ERR_UNSUPPORTED, "field must be real, integer or pattern");
    const bool mirrored = sym == "symmetric" || sym == "skew-symmetric";
    const double mirror_sign = sym == "skew-symmetric" ? -1.0 : 1.0;
    if (!mirrored && sym != "general") fail(ACC_SPMM_ERR_UNSUPPORTED, "symmetry must be general, symmetric or skew-symmetric");

    long long M = 0, K = 0, n = 0;
    for (;;) {  // comments and blank lines, then the size line
        if (!std::fgets(line.data(), (int)line.size(), f)) fail(ACC_SPMM_ERR_INVALID_ARG, "missing size line");
        const char* p = line.data();
        while (*p == ' ' || *p == '\t') ++p;
        if (*p == '%' || *p == '\n' || *p == '\r' || *p == 0) continue;
        if (std::sscanf(p, "%lld %lld %lld", &M, &K, &n) != 3) fail(ACC_SPMM_ERR_INVALID_ARG, "bad size line");
        break;
    }
    if (M < 0 || K < 0 || n < 0 || M >= (1ll << 31) || K >= (1ll << 31)) fail(ACC_SPMM_ERR_INVALID_ARG, "bad sizes");

    std::vector<Entry> entries;
    entries.reserve((size_t)(mirrored ? 2 * n : n));
    for (long long k = 0; k < n; ++k) {
        if (!std::fgets(line.data(), (int)line.size(), f)) fail(ACC_SPMM_ERR_INVALID_ARG, "fewer entries than the size line says");
        char* p = line.data();
        char* end = nullptr;
        const long long i = std::strtoll(p, &end, 10);
        if (end == p) {  // blank line inside the data: skip it
            --k;
            continue;
        }
        p = end;
        const long long j = std::strtoll(p, &end, 10);
        if (end == p) fail(ACC_SPMM_ERR_INVALID_ARG, "bad entry line");
        p = end;
        double v = 1.0;
        if (!pattern) {
            v = std::strtod(p, &end);
            if (end == p) fail(ACC_SPMM_ERR_INVALID_ARG, "entry without a value");
        }
        if (i < 1 || i > M || j < 1 || j > K) fail(ACC_SPMM_ERR_INVALID_ARG, "entry index outside the matrix");
        entries.push_back({(int32_t)(i - 1), (int32_t)(j - 1), v});
        if (mirrored && i != j) {
            if (j > M || i > K) fail(ACC_SPMM_ERR_INVALID_ARG, "symmetric file with a non-square shape");
            entries.push_back({(int32_t)(j - 1), (int32_t)(i - 1), mirror_sign * v});
        }
    }
    std::sort(entries.begin(), entries.end(), [](const Entry& a, const Entry& b) { return a.r != b.r ? a.r < b.r : a.c < b.c; });

    MtxFile* out = new MtxFile;
    try {
        out->M = M;
        out->K = K;
        out->rowptr.assign((size_t)M + 1, 0);
        for (size_t a = 0; a < entries.size();) {
            size_t b = a;
            double sum = 0.0;
            while (b < entries.size() && entries[b].r == entries[a].r && entries[b].c == entries[a].c) sum += entries[b++].v;
            out->colidx.push_back(entries[a].c);
            out->vals.push_back(value_type == ACC_SPMM_BF16 ? to_bf16_bits((float)sum) : to_half_bits((float)sum));
            ++out->rowptr[(size_t)entries[a].r + 1];
            a = b;
        }
        if (out->colidx.size() >= ((size_t)1 << 31)) fail(ACC_SPMM_ERR_UNSUPPORTED, "2^31 or more entries");
        for (long long r = 0; r < M; ++r) out->rowptr[(size_t)r + 1] += out->rowptr[(size_t)r];
    } catch (...) {
        delete out;
        throw;
    }
    return out;
}

void free_matrix_market(MtxFile* m) { delete m; }

void matrix_market_shape(const MtxFile* m, int64_t* M, int64_t* K, int64_t* nnz) {
    if (M) *M = m->M;
    if (K) *K = m->K;
    if (nnz) *nnz = (int64_t)m->colidx.size();
}

void matrix_market_csr(const MtxFile* m, int32_t* rowptr, int32_t* colidx, uint16_t* vals) {
    if (rowptr) std::memcpy(rowptr, m->rowptr.data(), m->rowptr.size() * sizeof(int32_t));
    if (colidx && !m->colidx.empty()) std::memcpy(colidx, m->colidx.data(), m->colidx.size() * sizeof(int32_t));
    if (vals && !m->vals.empty()) std::memcpy(vals, m->vals.data(), m->vals.size() * sizeof(uint16_t));
}

}  // namespace accspmm
