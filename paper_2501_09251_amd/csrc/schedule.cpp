// Adaptive sparsity-aware load balancing (paper Section 3.5): the imbalance degree of
// Eq. 3 and the distribution of tiles over work items guided by the cost model of Eq. 4.
//
// Reading of Eq. 4 (its printed load and write-back terms are identical and carry no byte
// sizes): a work item holding n tiles that closes s row windows costs
//     n * (TW*N*2/BW + 2*WH*TW*N/FLOPS)  +  s * (WH*N*4/BW)
// i.e. B rows loaded per tile, matrix-core time per tile, and one C write-back per window.
// N cancels out of every comparison, so the schedule does not depend on N.
#include <cmath>

#include "internal.h"

namespace accspmm {

double imbalance_degree(const std::vector<int32_t>& rwo) {
    const int64_t W = (int64_t)rwo.size() - 1;
    if (W <= 0) return 0.0;
    const double avg = (double)rwo[W] / (double)W;
    double s = 0.0;
    for (int64_t w = 0; w < W; ++w) s += std::fabs((double)(rwo[w + 1] - rwo[w]) - avg);
    return s / (double)W;
}

void build_schedule(const std::vector<int32_t>& rwo, bool balance, int32_t cap, int32_t WH, int32_t TW,
                    std::vector<WorkItem>& items, std::vector<SplitWindow>& splits, int64_t& n_slots) {
    const int64_t W = (int64_t)rwo.size() - 1;
    items.clear();
    splits.clear();
    n_slots = 0;
    if (!balance) {  // one work item per row window
        items.reserve(W);
        for (int64_t w = 0; w < W; ++w) items.push_back(WorkItem{(int32_t)w, (int32_t)w + 1, rwo[w], rwo[w + 1]});
        return;
    }
    // per-CU shares of the chip: 8 TB/s and 2.5 PFLOP/s (fp16 MFMA) over 256 CUs
    const double bw = 8.0e12 / 256.0, flops = 2.5e15 / 256.0;
    const double c_tile = TW * 2.0 / bw + 2.0 * WH * TW / flops;  // per feature column
    const double c_win = WH * 4.0 / bw;
    const double target = cap * c_tile + c_win;
    int64_t cur_begin = -1;
    double cur_cost = 0.0;
    auto close = [&](int64_t w_end) {
        if (cur_begin >= 0)
            items.push_back(WorkItem{(int32_t)cur_begin, (int32_t)w_end, rwo[cur_begin], rwo[w_end]});
        cur_begin = -1;
        cur_cost = 0.0;
    };
    for (int64_t w = 0; w < W; ++w) {
        const int32_t tw = rwo[w + 1] - rwo[w];
        if (tw > cap) {  // heavy window: split into near-equal slices, each with a partial slot
            close(w);
            const int32_t k = (tw + cap - 1) / cap;
            splits.push_back(SplitWindow{(int32_t)w, (int32_t)n_slots, (int32_t)(n_slots + k), 0});
            for (int32_t i = 0; i < k; ++i) {
                const int32_t b = rwo[w] + (int32_t)((int64_t)tw * i / k);
                const int32_t e = rwo[w] + (int32_t)((int64_t)tw * (i + 1) / k);
                items.push_back(WorkItem{(int32_t)w, (int32_t)(-(n_slots + i) - 1), b, e});
            }
            n_slots += k;
            continue;
        }
        const double c = tw * c_tile + c_win;
        if (cur_begin >= 0 && cur_cost + c > target) close(w);
        if (cur_begin < 0) cur_begin = w;
        cur_cost += c;
    }
    close(W);
}

}  // namespace accspmm
