// Driver for tests/test_host_sanitized.py: runs the host-only stages of the library (Step I of the
// reordering, the schedule, the Matrix Market reader) and the oracle on small seeded inputs in a
// build with AddressSanitizer and UndefinedBehaviorSanitizer.  Any report aborts the process.
#include <cstdio>
#include <cstdlib>
#include <random>
#include <algorithm>
#include <set>
#include <string>
#include <vector>

#include "internal.h"

namespace accspmm {
void fail(int code, const std::string& msg) { throw Failure{code, msg}; }
}  // namespace accspmm

extern "C" {
void orc_spmm_rows_typed(int64_t, const int64_t*, int64_t, const int32_t*, const int32_t*, const uint16_t*, const uint16_t*,
                         double*, double*, int);
void orc_sddmm(int64_t, int64_t, const int32_t*, const int32_t*, const uint16_t*, const uint16_t*, const uint16_t*, double*,
               double*, int);
int64_t orc_encode(int64_t, const int32_t*, const int32_t*, const uint16_t*, const int32_t*, int32_t, int32_t, int32_t*, int32_t*,
                   int32_t*, uint64_t*, uint16_t*);
double orc_ibd(int64_t, const int32_t*);
}

int main(int argc, char** argv) {
    using namespace accspmm;
    std::mt19937 rng(12345);
    for (int round = 0; round < 20; ++round) {
        // a random symmetric graph without self loops
        const int64_t M = 1 + rng() % 300;
        std::vector<std::set<int32_t>> nb(M);
        const int64_t edges = rng() % (3 * M + 1);
        for (int64_t e = 0; e < edges; ++e) {
            int32_t a = rng() % M, b = rng() % M;
            if (a != b) { nb[a].insert(b); nb[b].insert(a); }
        }
        std::vector<int64_t> gptr(M + 1, 0);
        std::vector<int32_t> gadj;
        for (int64_t i = 0; i < M; ++i) {
            for (int32_t j : nb[i]) gadj.push_back(j);
            gptr[i + 1] = (int64_t)gadj.size();
        }
        std::vector<int32_t> parent, seq;
        std::vector<int64_t> seg;
        double work = 0;
        const int32_t seg_len = 1 + rng() % 64;
        if (!build_dendrogram_host(M, gptr.data(), gadj.data(), seg_len, 0.0, parent, seq, seg, &work)) return 2;
        if ((int64_t)seq.size() != M || seg.back() != M) return 3;
        {   // the leaf sequence rebuilt from the parents and the visiting order (what follows the device form of
            // Step I) equals the one the host form produced itself
            std::vector<int32_t> order(M);
            for (int64_t i = 0; i < M; ++i) order[i] = (int32_t)i;
            std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
                return gptr[a + 1] - gptr[a] < gptr[b + 1] - gptr[b];
            });
            std::vector<int32_t> seq2;
            std::vector<int64_t> seg2;
            leaf_sequence_from_parents(M, parent, order, seg_len, seq2, seg2);
            if (seq2 != seq || seg2 != seg) return 6;
        }
        build_dendrogram_host(M, gptr.data(), gadj.data(), seg_len, 0.5, parent, seq, seg, &work);   // a budget that may stop it

        // a schedule over random tile counts, with a heavy window
        const int64_t W = 1 + rng() % 200;
        std::vector<int32_t> rwo(W + 1, 0);
        for (int64_t w = 0; w < W; ++w) rwo[w + 1] = rwo[w] + (rng() % 5 == 0 ? rng() % 400 : rng() % 6);
        std::vector<WorkItem> items;
        std::vector<SplitWindow> splits;
        int64_t slots = 0;
        build_schedule(rwo, rng() % 2, 1 + rng() % 64, 16, 16, items, splits, slots);
        int64_t covered = 0;
        for (const WorkItem& it : items) covered += it.t_end - it.t_begin;
        if (covered != rwo[W]) return 4;
        (void)imbalance_degree(rwo);

        // the oracle on the graph's pattern as a matrix
        std::vector<int32_t> rowptr(M + 1), colidx(gadj.begin(), gadj.end());
        for (int64_t i = 0; i <= M; ++i) rowptr[i] = (int32_t)gptr[i];
        const int64_t nnz = (int64_t)colidx.size(), N = 1 + rng() % 9;
        std::vector<uint16_t> vals(nnz), B(M * N), X(M * N);
        for (auto& v : vals) v = 0x3c00 + rng() % 512;
        for (auto& v : B) v = 0x3800 + rng() % 1024;
        for (auto& v : X) v = 0xb800 + rng() % 1024;
        std::vector<double> C(M * N), bound(M * N), out(nnz), ob(nnz);
        orc_spmm_rows_typed(M, nullptr, N, rowptr.data(), colidx.data(), vals.data(), B.data(), C.data(), bound.data(), round % 2);
        orc_sddmm(M, N, rowptr.data(), colidx.data(), vals.data(), X.data(), B.data(), out.data(), ob.data(), round % 2);
        const int64_t T = orc_encode(M, rowptr.data(), colidx.data(), vals.data(), nullptr, 16, 16, nullptr, nullptr, nullptr,
                                     nullptr, nullptr);
        if (T < 0) return 5;
        std::vector<int32_t> o_rwo((M + 15) / 16 + 1), o_tco(T + 1), o_a2b(T * 16);
        std::vector<uint64_t> o_bits(T * 4);
        std::vector<uint16_t> o_vals(nnz);
        orc_encode(M, rowptr.data(), colidx.data(), vals.data(), nullptr, 16, 16, o_rwo.data(), o_tco.data(), o_a2b.data(),
                   o_bits.data(), o_vals.data());
        (void)orc_ibd((int64_t)o_rwo.size() - 1, o_rwo.data());
    }
    // the Matrix Market reader on a good and on two broken files
    if (argc > 1) {
        const std::string dir = argv[1];
        auto write = [&](const char* name, const char* text) {
            std::FILE* f = std::fopen((dir + "/" + name).c_str(), "w");
            std::fputs(text, f);
            std::fclose(f);
        };
        write("ok.mtx", "%%MatrixMarket matrix coordinate real symmetric\n% c\n4 4 4\n1 1 2.5\n3 1 -1e-3\n4 2 7\n4 4 70000\n");
        write("short.mtx", "%%MatrixMarket matrix coordinate real general\n4 4 9\n1 1 2.5\n");
        write("range.mtx", "%%MatrixMarket matrix coordinate pattern general\n4 4 1\n5 1\n");
        MtxFile* m = read_matrix_market((dir + "/ok.mtx").c_str(), ACC_SPMM_FP16);
        int64_t M, K, nnz;
        matrix_market_shape(m, &M, &K, &nnz);
        std::vector<int32_t> rp(M + 1), ci(nnz);
        std::vector<uint16_t> va(nnz);
        matrix_market_csr(m, rp.data(), ci.data(), va.data());
        free_matrix_market(m);
        if (nnz != 6) return 6;
        for (const char* bad : {"short.mtx", "range.mtx", "missing.mtx"}) {
            try {
                free_matrix_market(read_matrix_market((dir + "/" + bad).c_str(), ACC_SPMM_BF16));
                return 7;
            } catch (const Failure&) {
            }
        }
    }
    std::puts("host stages clean");
    return 0;
}
