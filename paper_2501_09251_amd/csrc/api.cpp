// C ABI of the library (see include/acc_spmm.h): argument checks, plan orchestration,
// statistics and array export.  No exception leaves this file.
#include <algorithm>
#include <chrono>
#include <cstring>
#include <new>
#include <thread>

#include "internal.h"

namespace accspmm {

namespace {
thread_local int g_err_code = 0;
thread_local std::string g_err_msg;

double now_s() {
    using namespace std::chrono;
    return duration<double>(steady_clock::now().time_since_epoch()).count();
}

// Default cap on the tiles of one work item (Section 3.5 caps a thread block at 32 of its smaller
// tiles): about two rounds of work items over the machine's wave slots, between 32 and 1024.
// Swept on the two power-law workloads (tile + combine kernels): 0.89 M tiles, best at 128..192
// (0.577..0.592 ms against 0.611 at 256 and 0.647 at 512); 14.9 M tiles, best at 512..1024
// (8.20..8.36 ms against 8.47 at 256 and 8.56 at 2048).
constexpr int32_t kDefaultCapMin = 32, kDefaultCapMax = 1024, kDefaultCapHostStage = 256;
constexpr int64_t kWaveSlotsPerCu = 12, kItemRounds = 2;

int32_t default_cap(int64_t tiles, int compute_units) {
    const int64_t per_item = tiles / std::max<int64_t>(1, (int64_t)compute_units * kWaveSlotsPerCu * kItemRounds);
    return (int32_t)std::min<int64_t>(kDefaultCapMax, std::max<int64_t>(kDefaultCapMin, per_item));
}
// AUTO keeps the reordering only for >= 1 % fewer tiles.  Measured, reordered against input order:
// R-MAT 2^23 1.07 % fewer tiles, 3.6 % faster (fewer split windows); R-MAT 2^20 5.4 % fewer, 3 %
// faster; block model 55 % fewer, 2.3x faster; stencil 1.2 % fewer, 1.3 % slower (AUTO gives up on
// it earlier, on the work budget below).
constexpr double kAutoReorderMinGain = 0.01;
constexpr int32_t kDefaultSegLen = 1024;
constexpr float kDefaultIbdThreshold = 8.0f;
constexpr double kAutoReorderWorkBudget = 8.0;   // edge-record visits per graph entry
constexpr int64_t kHubSkewMinK = 65536;          // fewer columns: too few labels for the statistic
// AUTO column order only from 2^20 columns on.  Measured on unscrambled R-MAT inputs with B in
// the caller's order: the order pays once B exceeds about 256 MB, the size of the memory-side
// cache (+22..30 % at N >= 128 from 2^20 columns on; nothing at 2^19 columns and N = 128).  At
// N <= 64 the 64-bit addressing of the two-matrix gather costs more than the order gains below
// 2^22 columns (-12..-26 %, -4 % at 2^21), so below kDualEntriesMaxK columns the plan also keeps
// SparseAToB with plain input columns and execute reads all of B in place when N <= 64.
constexpr int64_t kAutoColumnOrderMinK = (int64_t)1 << 20;
constexpr int64_t kDualEntriesMaxK = (int64_t)1 << 22;
constexpr int64_t kHubSample = 65536;            // most used columns whose labels are examined
constexpr double kAutoColumnOrderSkew = 4.0;
// Rows of B gathered per execute when B comes in the caller's order: the first K/16 of the
// column order, at most 2^17.  Measured on R-MAT 2^23: moving the 2^14 most used columns gives
// most of the gain, 2^17 all of it (they carry 64 % of the entries), 2^20 nothing more.
constexpr int64_t kMaxHotColumns = (int64_t)1 << 17;

// How unevenly the labels of the most used columns (`top`, any order) fall on the residue
// classes modulo 16, 256 and 4096: the fullest class over an even share, the largest of the
// three moduli that leave at least 8 labels per class on average.  About 1 to 2 for labels
// unrelated to use counts; large when the heavy columns sit at power-of-two strides (the ids
// with few set bits of an unscrambled R-MAT graph), where their rows of B collide in the
// memory system.
double hub_label_skew(const std::vector<int32_t>& top) {
    double worst = 0.0;
    for (int bits : {4, 8, 12}) {
        const size_t classes = (size_t)1 << bits;
        if (top.size() < 8 * classes) continue;
        std::vector<int32_t> count(classes, 0);
        for (int32_t c : top) ++count[(size_t)c & (classes - 1)];
        const double even = (double)top.size() / (double)classes;
        worst = std::max(worst, (double)*std::max_element(count.begin(), count.end()) / even);
    }
    return worst;
}
}  // namespace

void set_error(int code, const std::string& msg) {
    g_err_code = code;
    g_err_msg = msg;
}

void fail(int code, const std::string& msg) { throw Failure{code, msg}; }

namespace {

// Checks the CSR (monotone row pointers, columns in range, no duplicate column in a row).
// Rows whose columns are not ascending are sorted into `fixed_*`; returns true if that
// copy must be used.  One pass over the entries, rows split over a few threads; the error
// reported is the one at the lowest row.
bool validate_csr(int64_t M, int64_t K, int64_t nnz, const int32_t* rowptr, const int32_t* colidx,
                  const uint16_t* vals, std::vector<int32_t>& fixed_col, std::vector<uint16_t>& fixed_val) {
    if (rowptr[0] != 0) fail(ACC_SPMM_ERR_INVALID_CSR, "csr_rowptr[0] must be 0");
    for (int64_t i = 0; i < M; ++i)
        if (rowptr[i + 1] < rowptr[i]) fail(ACC_SPMM_ERR_INVALID_CSR, "csr_rowptr decreases at row " + std::to_string(i));
    if (rowptr[M] != nnz) fail(ACC_SPMM_ERR_INVALID_CSR, "csr_rowptr[M] != nnz");
    struct Finding {
        int64_t bad_entry = -1;   // first entry whose column is out of range
        bool unsorted = false;    // some row's columns are not strictly ascending
    };
    const int n_threads = nnz < (1 << 22) ? 1 : (int)std::min<unsigned>(16u, std::max(1u, std::thread::hardware_concurrency()));
    std::vector<Finding> found(n_threads);
    auto scan = [&](int k) {
        // rows [r0, r1): equal shares of the entries
        const int64_t e0 = nnz * k / n_threads, e1 = nnz * (k + 1) / n_threads;
        const int64_t r0 = k == 0 ? 0 : std::upper_bound(rowptr, rowptr + M + 1, (int32_t)e0) - rowptr - 1;
        const int64_t r1 = k == n_threads - 1 ? M : std::upper_bound(rowptr, rowptr + M + 1, (int32_t)e1) - rowptr - 1;
        Finding f;
        for (int64_t i = r0; i < r1 && f.bad_entry < 0; ++i) {
            const int64_t b = rowptr[i], e = rowptr[i + 1];
            for (int64_t p = b; p < e; ++p) {
                const int32_t c = colidx[p];
                if (c < 0 || c >= K) { f.bad_entry = p; break; }
                if (p > b && c <= colidx[p - 1]) f.unsorted = true;
            }
        }
        found[k] = f;
    };
    if (n_threads == 1) {
        scan(0);
    } else {
        std::vector<std::thread> pool;
        for (int k = 0; k < n_threads; ++k) pool.emplace_back(scan, k);
        for (auto& th : pool) th.join();
    }
    bool unsorted = false;
    for (const Finding& f : found) {
        if (f.bad_entry >= 0) fail(ACC_SPMM_ERR_INVALID_CSR, "column index out of range at entry " + std::to_string(f.bad_entry));
        unsorted = unsorted || f.unsorted;
    }
    if (!unsorted) return false;   // strictly ascending everywhere: no duplicates either
    fixed_col.assign(colidx, colidx + nnz);
    fixed_val.assign(vals, vals + nnz);
    std::vector<std::pair<int32_t, uint16_t>> row;
    for (int64_t i = 0; i < M; ++i) {
        const int64_t b = rowptr[i], e = rowptr[i + 1];
        if (!std::is_sorted(colidx + b, colidx + e)) {
            row.clear();
            for (int64_t p = b; p < e; ++p) row.push_back({colidx[p], vals[p]});
            std::stable_sort(row.begin(), row.end(), [](auto& x, auto& y) { return x.first < y.first; });
            for (int64_t p = b; p < e; ++p) { fixed_col[p] = row[p - b].first; fixed_val[p] = row[p - b].second; }
        }
        for (int64_t p = b + 1; p < e; ++p)
            if (fixed_col[p] == fixed_col[p - 1])
                fail(ACC_SPMM_ERR_INVALID_CSR, "duplicate column " + std::to_string(fixed_col[p]) + " in row " + std::to_string(i));
    }
    return true;
}

// The graph build of the reordering numbers the 2*nnz directed edge keys, and their run heads,
// with 32-bit positions: beyond this many entries the reordering is not available (ON is
// refused, AUTO keeps the input order).
constexpr int64_t kReorderMaxNnz = ((int64_t)1 << 30) - 1;

struct RowOrderInfo {
    bool applied = false;
    int64_t tiles_identity = -1;   // tile count in the input order, if it was counted
    double work_ratio = 0.0, t_graph = 0.0, t_dendrogram = 0.0, t_ordering = 0.0, t_total = 0.0;
    bool on_device = false;        // Step I ran in its device form
    int64_t rounds = 0;            // rounds of that form
};

// Row order of the plan (Section 3.2): d_perm / P.perm / P.iperm get the data-affinity order if
// the options ask for it and, under AUTO, it pays; else the identity.
void choose_row_order(Plan& P, int64_t M, int64_t K, int64_t nnz, const int32_t* rowptr, DevBuf<int32_t>& d_perm,
                      RowOrderInfo& info) {
    const acc_spmm_options& opt = P.opt;
    const int32_t WH = opt.window_height, TW = opt.tile_width;
    std::vector<int32_t> identity(M);
    for (int64_t i = 0; i < M; ++i) identity[i] = (int32_t)i;
    d_perm.upload(identity.data(), M);
    if (opt.reorder != ACC_SPMM_OFF && M == K && M > 0 && nnz > 0 && nnz <= kReorderMaxNnz) {
        const double r0 = now_s();
        // AUTO gives up on inputs whose dendrogram is expensive to build (large uniform
        // meshes), where the identity order is kept anyway; ON always completes.
        const double budget = opt.reorder == ACC_SPMM_AUTO ? kAutoReorderWorkBudget : 0.0;
        std::vector<int32_t> seq;
        std::vector<int64_t> seg_start;
        bool complete;
        {
            const double g0 = now_s();
            DeviceGraph graph;
            build_graph_on_device(M, nnz, P.d_rowptr.p, P.d_colidx.p, graph);
            const double g1 = now_s();
            // Step I on the GPU; its host form takes over if the device form reports that this input
            // does not suit it (memory pools exhausted, or rounds that advance by a few vertices only)
            std::vector<int32_t> order;
            int how = opt.dendrogram_on_host ? kDendrogramUseHost
                                             : build_dendrogram_on_device(graph, budget, P.parent, order, &info.work_ratio, &info.rounds);
            if (how == kDendrogramUseHost) {
                HostGraph host_graph;
                copy_graph_to_host(graph, host_graph);
                graph.adj.release();
                graph.ptr.release();
                info.on_device = false;
                complete = build_dendrogram_host(M, host_graph.ptr, host_graph.adj, opt.segment_length, budget, P.parent, seq,
                                                 seg_start, &info.work_ratio);
            } else {
                info.on_device = true;
                complete = how == kDendrogramDone;
                if (complete) leaf_sequence_from_parents(M, P.parent, order, opt.segment_length, seq, seg_start);
            }
            info.t_graph = g1 - g0;
            info.t_dendrogram = now_s() - g1;
        }
        if (!complete) {
            P.parent.clear();
        } else {
            const double o0 = now_s();
            int32_t max_row_len = 0;
            for (int64_t i = 0; i < M; ++i) max_row_len = std::max(max_row_len, rowptr[i + 1] - rowptr[i]);
            DevBuf<int32_t> d_new;
            ordering_on_device(M, K, nnz, P.d_rowptr.p, P.d_colidx.p, seq, seg_start, opt.segment_length, max_row_len, d_new);
            info.t_ordering = now_s() - o0;
            DeviceFormat probe;
            encode_on_device(M, K, nnz, P.d_rowptr.p, P.d_colidx.p, P.d_vals.p, d_perm.p, WH, TW, probe, true);
            info.tiles_identity = probe.T;
            encode_on_device(M, K, nnz, P.d_rowptr.p, P.d_colidx.p, P.d_vals.p, d_new.p, WH, TW, probe, true);
            info.applied = opt.reorder == ACC_SPMM_ON ||
                           (double)probe.T <= (1.0 - kAutoReorderMinGain) * (double)info.tiles_identity;
            if (info.applied) {
                P.perm.resize(M);
                d_new.download(P.perm.data());
                P.iperm.resize(M);
                for (int64_t r = 0; r < M; ++r) P.iperm[P.perm[r]] = (int32_t)r;
                ACC_HIP(hipMemcpy(d_perm.p, d_new.p, sizeof(int32_t) * M, hipMemcpyDeviceToDevice));
            }
        }
        info.t_total = now_s() - r0;
    }
    if (!info.applied) {
        P.perm = identity;
        P.iperm = std::move(identity);
    }
}

// Column order of the plan: when the options ask for one and, under AUTO, the labels of the
// most used columns call for it, P.d_col_order / col_order / col_rank are filled and
// d_colidx_plan gets the column indices relabelled into it; else everything stays empty.
void choose_column_order(Plan& P, int64_t K, int64_t nnz, DevBuf<int32_t>& d_colidx_plan, double& skew) {
    const acc_spmm_options& opt = P.opt;
    skew = 0.0;
    if (opt.column_order == ACC_SPMM_OFF || K == 0 || nnz == 0) return;
    if (opt.column_order == ACC_SPMM_AUTO && K < kHubSkewMinK) return;   // too small for AUTO to ever apply
    DevBuf<int32_t> d_order, d_rank;
    column_order_on_device(K, nnz, P.d_colidx.p, d_order, d_rank);
    if (K >= kHubSkewMinK) {
        std::vector<int32_t> top((size_t)std::min<int64_t>(kHubSample, K / 16));
        ACC_HIP(hipMemcpy(top.data(), d_order.p, sizeof(int32_t) * top.size(), hipMemcpyDeviceToHost));
        skew = hub_label_skew(top);
    }
    const bool apply = opt.column_order == ACC_SPMM_ON || (K >= kAutoColumnOrderMinK && skew >= kAutoColumnOrderSkew);
    if (!apply) return;
    P.col_order.resize(K);
    P.col_rank.resize(K);
    d_order.download(P.col_order.data());
    d_rank.download(P.col_rank.data());
    d_colidx_plan.alloc(nnz);
    remap_columns_on_device(nnz, P.d_colidx.p, d_rank.p, d_colidx_plan.p);
    P.d_col_order.swap(d_order);
}

acc_spmm_plan_t* build_plan(int64_t M, int64_t K, int64_t nnz, const int32_t* rowptr, const int32_t* colidx,
                            const uint16_t* vals, const acc_spmm_options* user) {
    const double t0 = now_s();
    if (M < 0 || K < 0 || nnz < 0 || M >= ((int64_t)1 << 31) || K >= ((int64_t)1 << 31) || nnz >= ((int64_t)1 << 31))
        fail(ACC_SPMM_ERR_INVALID_ARG, "M, K and nnz must be in [0, 2^31)");
    if (!rowptr || (nnz > 0 && (!colidx || !vals))) fail(ACC_SPMM_ERR_INVALID_ARG, "null CSR pointer");
    acc_spmm_options opt{};
    opt.reorder = ACC_SPMM_AUTO;
    opt.load_balance = ACC_SPMM_AUTO;
    opt.column_order = ACC_SPMM_AUTO;
    if (user) {
        if (user->struct_size != (int32_t)sizeof(acc_spmm_options))
            fail(ACC_SPMM_ERR_INVALID_ARG, "options.struct_size does not match this library");
        opt = *user;
    }
    if (opt.column_order < 0 || opt.column_order > 2) fail(ACC_SPMM_ERR_INVALID_ARG, "column_order must be OFF, ON or AUTO");
    if (opt.operand_order < 0 || opt.operand_order > 1) fail(ACC_SPMM_ERR_INVALID_ARG, "operand_order must be 0 or 1");
    if (opt.reorder < 0 || opt.reorder > 2 || opt.load_balance < 0 || opt.load_balance > 2)
        fail(ACC_SPMM_ERR_INVALID_ARG, "reorder / load_balance must be OFF, ON or AUTO");
    if (opt.window_height == 0) opt.window_height = 16;
    if (opt.tile_width == 0) opt.tile_width = 16;
    {
        const int32_t wh = opt.window_height, tw = opt.tile_width;
        const bool ok = (wh == 8 || wh == 16 || wh == 32 || wh == 64) && (tw == 8 || tw == 16 || tw == 32);
        if (!ok) fail(ACC_SPMM_ERR_UNSUPPORTED, "window_height must be 8, 16, 32 or 64 and tile_width 8, 16 or 32");
    }
    if (opt.max_tiles_per_item < 0) fail(ACC_SPMM_ERR_INVALID_ARG, "max_tiles_per_item must not be negative");
    if (opt.segment_length == 0) opt.segment_length = kDefaultSegLen;
    if (opt.segment_length < 1) fail(ACC_SPMM_ERR_INVALID_ARG, "segment_length must be positive");
    if (opt.ibd_threshold == 0.f) opt.ibd_threshold = kDefaultIbdThreshold;
    if (opt.pipeline_depth < 0 || opt.pipeline_depth > 3) fail(ACC_SPMM_ERR_INVALID_ARG, "pipeline_depth must be 0..3");
    if (opt.value_fetch < 0 || opt.value_fetch > 3) fail(ACC_SPMM_ERR_INVALID_ARG, "value_fetch must be 0, 1, 2 or 3");
    if (opt.dendrogram_on_host < 0 || opt.dendrogram_on_host > 1) fail(ACC_SPMM_ERR_INVALID_ARG, "dendrogram_on_host must be 0 or 1");
    if (opt.lds_staging < 0 || opt.lds_staging > 1) fail(ACC_SPMM_ERR_INVALID_ARG, "lds_staging must be 0 or 1");
    if (opt.slabs_per_wave < 0 || opt.slabs_per_wave > 2) fail(ACC_SPMM_ERR_INVALID_ARG, "slabs_per_wave must be 0, 1 or 2");
    if (opt.value_type != ACC_SPMM_FP16 && opt.value_type != ACC_SPMM_BF16)
        fail(ACC_SPMM_ERR_INVALID_ARG, "value_type must be ACC_SPMM_FP16 or ACC_SPMM_BF16");

    if (opt.reorder == ACC_SPMM_ON && M == K && nnz > kReorderMaxNnz)
        fail(ACC_SPMM_ERR_UNSUPPORTED, "reorder = ON needs nnz < 2^30 (the pattern graph is indexed with 32 bits); "
                                       "use reorder = AUTO or OFF, which keep the input order for such a matrix");

    std::vector<int32_t> fixed_col;
    std::vector<uint16_t> fixed_val;
    if (validate_csr(M, K, nnz, rowptr, colidx, vals, fixed_col, fixed_val)) {
        colidx = fixed_col.data();
        vals = fixed_val.data();
    }

    int dev_count = 0;
    if (hipGetDeviceCount(&dev_count) != hipSuccess || dev_count == 0)
        fail(ACC_SPMM_ERR_HIP, "no HIP device: this library only runs on a gfx950 GPU (there is no CPU path)");
    const double t1 = now_s();

    acc_spmm_plan_t* handle = new acc_spmm_plan_t;
    Plan& P = handle->plan;
    try {
        ACC_HIP(hipGetDevice(&P.device));
        prepare_static_scratch();
        P.opt = opt;
        const int32_t WH = opt.window_height, TW = opt.tile_width;

        // device copy of the CSR
        P.d_rowptr.upload(rowptr, M + 1);
        P.d_colidx.upload(colidx, nnz);
        P.d_vals.upload(vals, nnz);

        // ---- row order ----
        DevBuf<int32_t> d_perm;
        RowOrderInfo ro;
        choose_row_order(P, M, K, nnz, rowptr, d_perm, ro);

        // ---- column order ----
        const double c0 = now_s();
        double skew = 0.0;
        DevBuf<int32_t> d_colidx_plan;   // column indices in the plan's column order (only if one is applied)
        choose_column_order(P, K, nnz, d_colidx_plan, skew);
        const bool use_col_order = P.d_col_order.p != nullptr;
        const double t_col_order = now_s() - c0;

        // ---- format ----
        const double e0 = now_s();
        encode_on_device(M, K, nnz, P.d_rowptr.p, use_col_order ? d_colidx_plan.p : P.d_colidx.p, P.d_vals.p, d_perm.p, WH,
                         TW, P.fmt, false, opt.keep_entry_map ? &P.d_entry_of : nullptr);
        const double t_encode = now_s() - e0;
        // the comparison kernel reads B as execute is given it
        if (use_col_order && opt.operand_order == 1 && opt.keep_csr) P.d_colidx.swap(d_colidx_plan);
        d_colidx_plan.release();
        if (use_col_order && opt.operand_order == 0) {
            // B stays in the caller's order: only the most used rows are gathered per call
            P.n_hot = (int32_t)std::min<int64_t>(kMaxHotColumns, K / 16);
            // below kDualEntriesMaxK columns whether the gathered copy pays depends on N, known only
            // at execute: keep the entries in both forms there
            if (K < kDualEntriesMaxK) P.a2b_plain.alloc((size_t)(P.fmt.T * TW));
            hot_cold_entries_on_device(P.fmt.T * TW, P.fmt.sparse_a_to_b.p, P.d_col_order.p, P.n_hot, P.a2b_plain.p);
        }
        if (!opt.keep_csr) {
            P.d_rowptr.release();
            P.d_colidx.release();
            P.d_vals.release();
        }

        // ---- schedule ----
        const double s0 = now_s();
        const int64_t W = P.fmt.W;
        std::vector<int32_t> rwo(W + 1, 0);
        P.fmt.row_window_offset.download(rwo.data());
        const double ibd = imbalance_degree(rwo);
        const bool balance = opt.load_balance == ACC_SPMM_ON || (opt.load_balance == ACC_SPMM_AUTO && ibd > opt.ibd_threshold);
        if (opt.max_tiles_per_item == 0) {
            int cus = 0;
            ACC_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, P.device));
            P.opt.max_tiles_per_item = default_cap(P.fmt.T, cus);
        }
        build_schedule(rwo, balance, P.opt.max_tiles_per_item, WH, TW, P.items, P.splits, P.n_slots);
        P.d_items.upload(P.items.data(), P.items.size());
        P.d_splits.upload(P.splits.data(), P.splits.size());
        std::vector<int32_t> pad((size_t)W * WH, -1);
        std::copy(P.perm.begin(), P.perm.end(), pad.begin());
        P.d_perm_pad.upload(pad.data(), pad.size());
        const double t_schedule = now_s() - s0;

        // ---- statistics ----
        acc_spmm_stats& st = P.stats;
        st.M = M; st.K = K; st.nnz = nnz;
        st.window_height = WH; st.tile_width = TW;
        st.num_windows = W;
        st.num_tiles = P.fmt.T;
        st.sum_distinct_cols = P.fmt.sum_dw;
        st.num_tiles_identity = ro.tiles_identity >= 0 ? ro.tiles_identity : P.fmt.T;
        st.num_items = (int64_t)P.items.size();
        st.num_split_windows = (int64_t)P.splits.size();
        st.num_partial_slots = P.n_slots;
        st.max_tiles_per_item = P.opt.max_tiles_per_item;
        st.reorder_applied = ro.applied;
        st.load_balance_applied = balance;
        st.ibd = ibd;
        st.mean_nnz_per_tile = P.fmt.T ? (double)nnz / (double)P.fmt.T : 0.0;
        st.index_bytes = 4 * (W + 1) + 4 * (P.fmt.T + 1) + 4 * P.fmt.T * TW + 8 * P.fmt.T * P.fmt.NW;
        st.schedule_bytes = (int64_t)(sizeof(WorkItem) * P.items.size() + sizeof(SplitWindow) * P.splits.size()) + 4 * W * WH;
        st.reorder_work_ratio = ro.work_ratio;
        st.t_graph_s = ro.t_graph;
        st.t_dendrogram_s = ro.t_dendrogram;
        st.dendrogram_on_device = ro.on_device;
        st.dendrogram_rounds = ro.rounds;
        st.t_ordering_s = ro.t_ordering;
        st.t_validate_s = t1 - t0;
        st.t_reorder_s = ro.t_total;
        st.t_encode_s = t_encode;
        st.t_schedule_s = t_schedule;
        st.column_order_applied = use_col_order;
        st.num_hot_columns = P.n_hot;
        st.hub_label_skew = skew;
        st.t_column_order_s = t_col_order;
        st.t_total_s = now_s() - t0;
    } catch (...) {
        delete handle;
        throw;
    }
    return handle;
}

template <class F>
int guarded(F&& fn) {
    try {
        fn();
        return ACC_SPMM_OK;
    } catch (const Failure& f) {
        set_error(f.code, f.msg);
        return f.code;
    } catch (const std::bad_alloc&) {
        set_error(ACC_SPMM_ERR_OOM, "host allocation failed");
        return ACC_SPMM_ERR_OOM;
    } catch (const std::exception& e) {
        set_error(ACC_SPMM_ERR_INVALID_ARG, e.what());
        return ACC_SPMM_ERR_INVALID_ARG;
    } catch (...) {   // nothing may leave through the C boundary
        set_error(ACC_SPMM_ERR_INVALID_ARG, "unknown failure");
        return ACC_SPMM_ERR_INVALID_ARG;
    }
}

}  // namespace
}  // namespace accspmm

using namespace accspmm;

extern "C" {

acc_spmm_plan_t* acc_spmm_plan_ex(int64_t M, int64_t K, int64_t nnz, const int32_t* csr_rowptr,
                                  const int32_t* csr_colidx, const uint16_t* csr_vals,
                                  const acc_spmm_options* options) {
    acc_spmm_plan_t* out = nullptr;
    guarded([&] { out = build_plan(M, K, nnz, csr_rowptr, csr_colidx, csr_vals, options); });
    return out;
}

acc_spmm_plan_t* acc_spmm_plan_device(int64_t M, int64_t K, int64_t nnz, const int32_t* csr_rowptr,
                                      const int32_t* csr_colidx, const uint16_t* csr_vals,
                                      const acc_spmm_options* options) {
    acc_spmm_plan_t* out = nullptr;
    guarded([&] {
        if (M < 0 || nnz < 0 || M >= ((int64_t)1 << 31) || nnz >= ((int64_t)1 << 31))
            fail(ACC_SPMM_ERR_INVALID_ARG, "M, K and nnz must be in [0, 2^31)");
        if (!csr_rowptr || (nnz > 0 && (!csr_colidx || !csr_vals))) fail(ACC_SPMM_ERR_INVALID_ARG, "null CSR pointer");
        // the plan validates and reorders on the host: bring the arrays over, then proceed as for host input
        std::vector<int32_t> rowptr((size_t)M + 1), colidx((size_t)nnz);
        std::vector<uint16_t> vals((size_t)nnz);
        ACC_HIP(hipMemcpy(rowptr.data(), csr_rowptr, rowptr.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
        if (nnz > 0) {
            ACC_HIP(hipMemcpy(colidx.data(), csr_colidx, colidx.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
            ACC_HIP(hipMemcpy(vals.data(), csr_vals, vals.size() * sizeof(uint16_t), hipMemcpyDeviceToHost));
        }
        out = build_plan(M, K, nnz, rowptr.data(), colidx.data(), vals.data(), options);
    });
    return out;
}

acc_spmm_plan_t* acc_spmm_plan(int64_t M, int64_t K, int64_t nnz, const int32_t* csr_rowptr,
                               const int32_t* csr_colidx, const uint16_t* csr_vals) {
    return acc_spmm_plan_ex(M, K, nnz, csr_rowptr, csr_colidx, csr_vals, nullptr);
}

int acc_spmm_execute(const acc_spmm_plan_t* plan, const void* B, int32_t N, void* C, void* stream) {
    return guarded([&] {
        if (!plan || !C || (!B && plan->plan.fmt.nnz > 0)) fail(ACC_SPMM_ERR_INVALID_ARG, "null argument");
        launch_execute(plan->plan, B, N, C, static_cast<hipStream_t>(stream));
    });
}

int acc_spmm_execute_c16(const acc_spmm_plan_t* plan, const void* B, int32_t N, void* C, void* stream) {
    return guarded([&] {
        if (!plan || !C || (!B && plan->plan.fmt.nnz > 0)) fail(ACC_SPMM_ERR_INVALID_ARG, "null argument");
        launch_execute(plan->plan, B, N, C, static_cast<hipStream_t>(stream), nullptr, nullptr, nullptr, true);
    });
}

int acc_spmm_execute_static(const acc_spmm_plan_t* plan, const void* B, int32_t N, void* C, void* stream) {
    return guarded([&] {
        if (!plan || !C || (!B && plan->plan.fmt.nnz > 0)) fail(ACC_SPMM_ERR_INVALID_ARG, "null argument");
        launch_execute(plan->plan, B, N, C, static_cast<hipStream_t>(stream), nullptr, nullptr, nullptr, false, true);
    });
}

int acc_spmm_execute_timed(const acc_spmm_plan_t* plan, const void* B, int32_t N, void* C, void* stream,
                           float* tiles_ms, float* combine_ms, float* gather_ms) {
    return guarded([&] {
        if (!plan || !C || !tiles_ms || (!B && plan->plan.fmt.nnz > 0)) fail(ACC_SPMM_ERR_INVALID_ARG, "null argument");
        launch_execute(plan->plan, B, N, C, static_cast<hipStream_t>(stream), tiles_ms, combine_ms, gather_ms);
    });
}

int acc_spmm_sddmm(const acc_spmm_plan_t* plan, const void* X, const void* Y, int32_t N, void* out, int32_t use_values,
                   void* stream) {
    return guarded([&] {
        if (!plan || ((!X || !Y || !out) && plan->plan.fmt.nnz > 0)) fail(ACC_SPMM_ERR_INVALID_ARG, "null argument");
        launch_sddmm(plan->plan, X, Y, N, out, use_values != 0, static_cast<hipStream_t>(stream));
    });
}

int acc_spmm_update_values(acc_spmm_plan_t* plan, const void* csr_vals, void* stream) {
    return guarded([&] {
        if (!plan || (!csr_vals && plan->plan.fmt.nnz > 0)) fail(ACC_SPMM_ERR_INVALID_ARG, "null argument");
        launch_update_values(plan->plan, csr_vals, static_cast<hipStream_t>(stream));
    });
}

int acc_spmm_permute_rows(const acc_spmm_plan_t* plan, const void* src, void* dst, int64_t row_bytes, int32_t to_caller,
                          void* stream) {
    return guarded([&] {
        if (!plan || !src || !dst) fail(ACC_SPMM_ERR_INVALID_ARG, "null argument");
        if (row_bytes <= 0 || (row_bytes & 1)) fail(ACC_SPMM_ERR_INVALID_ARG, "row_bytes must be a positive multiple of 2");
        const Plan& P = plan->plan;
        int dev = -1;
        ACC_HIP(hipGetDevice(&dev));
        if (dev != P.device) fail(ACC_SPMM_ERR_INVALID_ARG, "the plan lives on another device than the current one");
        if (P.stats.K == 0) return;
        if (!P.d_col_order.p) {
            ACC_HIP(hipMemcpyAsync(dst, src, (size_t)P.stats.K * (size_t)row_bytes, hipMemcpyDeviceToDevice,
                                   static_cast<hipStream_t>(stream)));
            return;
        }
        launch_permute_rows(P.d_col_order.p, P.stats.K, src, dst, row_bytes, to_caller != 0, static_cast<hipStream_t>(stream));
    });
}

int acc_spmm_execute_csr_naive(const acc_spmm_plan_t* plan, const void* B, int32_t N, void* C, void* stream) {
    return guarded([&] {
        if (!plan || !C || (!B && plan->plan.fmt.nnz > 0)) fail(ACC_SPMM_ERR_INVALID_ARG, "null argument");
        launch_csr_naive(plan->plan, B, N, C, static_cast<hipStream_t>(stream));
    });
}

void acc_spmm_destroy(acc_spmm_plan_t* plan) { delete plan; }

int acc_spmm_plan_save(const acc_spmm_plan_t* plan, const char* path) {
    return guarded([&] {
        if (!plan) fail(ACC_SPMM_ERR_INVALID_ARG, "null argument");
        save_plan(plan->plan, path);
    });
}

acc_spmm_plan_t* acc_spmm_plan_load(const char* path) {
    acc_spmm_plan_t* out = nullptr;
    guarded([&] { out = load_plan(path); });
    return out;
}

int acc_spmm_last_error(char* buf, size_t len) {
    if (buf && len) {
        std::strncpy(buf, g_err_msg.c_str(), len - 1);
        buf[len - 1] = 0;
    }
    return g_err_code;
}

int acc_spmm_plan_stats(const acc_spmm_plan_t* plan, acc_spmm_stats* out) {
    return guarded([&] {
        if (!plan || !out) fail(ACC_SPMM_ERR_INVALID_ARG, "null argument");
        *out = plan->plan.stats;
    });
}

int acc_spmm_plan_traffic(const acc_spmm_plan_t* plan, int32_t N, int64_t* a_bytes, int64_t* b_bytes,
                          int64_t* c_bytes, int64_t* mfma_flops) {
    return guarded([&] {
        if (!plan || N <= 0) fail(ACC_SPMM_ERR_INVALID_ARG, "bad argument");
        const acc_spmm_stats& st = plan->plan.stats;
        if (a_bytes) *a_bytes = 2 * st.nnz + st.index_bytes + st.schedule_bytes;
        if (b_bytes) *b_bytes = st.sum_distinct_cols * (int64_t)N * 2;
        if (c_bytes) *c_bytes = st.M * (int64_t)N * 4;
        if (mfma_flops) *mfma_flops = 2 * st.num_tiles * st.window_height * st.tile_width * (int64_t)N;
    });
}

int acc_spmm_calibration_copy(void* dst, const void* src, size_t bytes, void* stream) {
    return guarded([&] { launch_calibration_copy(dst, src, bytes, static_cast<hipStream_t>(stream)); });
}

int acc_spmm_calibration_gather(const void* table, int64_t rows, int64_t row_bytes, const int32_t* index, int64_t n_index,
                                void* sink, size_t sink_bytes, void* out, size_t out_bytes, int32_t write_every,
                                int32_t write_rows, void* stream) {
    return guarded([&] {
        launch_calibration_gather(table, rows, row_bytes, index, n_index, sink, sink_bytes, out, out_bytes, write_every,
                                  write_rows, static_cast<hipStream_t>(stream));
    });
}

int64_t acc_spmm_dendrogram_host(int64_t M, const int64_t* graph_rowptr, const int32_t* graph_adj,
                                 int32_t segment_length, int32_t* parent, int32_t* leaf_sequence,
                                 int32_t* segment_start, double* work_ratio) {
    int64_t nseg = -1;
    int rc = guarded([&] {
        if (M < 0 || M >= ((int64_t)1 << 31) || !graph_rowptr || !parent) fail(ACC_SPMM_ERR_INVALID_ARG, "bad argument");
        if (graph_rowptr[0] != 0) fail(ACC_SPMM_ERR_INVALID_CSR, "graph_rowptr[0] must be 0");
        for (int64_t i = 0; i < M; ++i) {
            if (graph_rowptr[i + 1] < graph_rowptr[i]) fail(ACC_SPMM_ERR_INVALID_CSR, "graph_rowptr decreases");
            for (int64_t p = graph_rowptr[i]; p < graph_rowptr[i + 1]; ++p) {
                const int32_t j = graph_adj[p];
                if (j < 0 || j >= M || j == i || (p > graph_rowptr[i] && j <= graph_adj[p - 1]))
                    fail(ACC_SPMM_ERR_INVALID_CSR, "neighbours must be ascending, in range and without self loops");
            }
        }
        std::vector<int32_t> par, seq;
        std::vector<int64_t> seg;
        build_dendrogram_host(M, graph_rowptr, graph_adj, segment_length > 0 ? segment_length : kDefaultSegLen, 0.0, par,
                              seq, seg, work_ratio);
        std::copy(par.begin(), par.end(), parent);
        if (leaf_sequence) std::copy(seq.begin(), seq.end(), leaf_sequence);
        if (segment_start) for (size_t i = 0; i < seg.size(); ++i) segment_start[i] = (int32_t)seg[i];
        nseg = (int64_t)seg.size() - 1;
    });
    return rc == ACC_SPMM_OK ? nseg : rc;
}

int64_t acc_spmm_schedule_host(int64_t W, const int32_t* row_window_offset, int32_t load_balance,
                               int32_t max_tiles_per_item, float ibd_threshold, double* ibd_out,
                               int32_t* items, int64_t items_capacity, int64_t* num_partial_slots) {
    int64_t n = -1;
    int rc = guarded([&] {
        if (W < 0 || !row_window_offset || load_balance < 0 || load_balance > 2)
            fail(ACC_SPMM_ERR_INVALID_ARG, "bad argument");
        std::vector<int32_t> rwo(row_window_offset, row_window_offset + W + 1);
        const double ibd = imbalance_degree(rwo);
        if (ibd_out) *ibd_out = ibd;
        const float thr = ibd_threshold > 0.f ? ibd_threshold : kDefaultIbdThreshold;
        const bool balance = load_balance == ACC_SPMM_ON || (load_balance == ACC_SPMM_AUTO && ibd > thr);
        std::vector<WorkItem> it;
        std::vector<SplitWindow> sp;
        int64_t slots = 0;
        build_schedule(rwo, balance, max_tiles_per_item > 0 ? max_tiles_per_item : kDefaultCapHostStage, 16, 16, it, sp, slots);
        if (num_partial_slots) *num_partial_slots = slots;
        if (items) {
            if ((int64_t)it.size() > items_capacity) fail(ACC_SPMM_ERR_INVALID_ARG, "items_capacity too small");
            std::memcpy(items, it.data(), it.size() * sizeof(WorkItem));
        }
        n = (int64_t)it.size();
    });
    return rc == ACC_SPMM_OK ? n : rc;
}

int acc_spmm_plan_export(const acc_spmm_plan_t* plan, int which, void* host_dst, size_t* bytes) {
    return guarded([&] {
        if (!plan || !bytes) fail(ACC_SPMM_ERR_INVALID_ARG, "null argument");
        const Plan& P = plan->plan;
        const DeviceFormat& f = P.fmt;
        const void* dev = nullptr;
        const void* host = nullptr;
        size_t need = 0;
        switch (which) {
            case ACC_SPMM_ARR_PERM: host = P.perm.data(); need = P.perm.size() * 4; break;
            case ACC_SPMM_ARR_IPERM: host = P.iperm.data(); need = P.iperm.size() * 4; break;
            case ACC_SPMM_ARR_DENDROGRAM_PARENT: host = P.parent.data(); need = P.parent.size() * 4; break;
            case ACC_SPMM_ARR_COL_ORDER: host = P.col_order.data(); need = P.col_order.size() * 4; break;
            case ACC_SPMM_ARR_COL_RANK: host = P.col_rank.data(); need = P.col_rank.size() * 4; break;
            case ACC_SPMM_ARR_WORK_ITEMS: host = P.items.data(); need = P.items.size() * sizeof(WorkItem); break;
            case ACC_SPMM_ARR_ROW_WINDOW_OFFSET: dev = f.row_window_offset.p; need = (size_t)(f.W + 1) * 4; break;
            case ACC_SPMM_ARR_TC_OFFSET: dev = f.tc_offset.p; need = (size_t)(f.T + 1) * 4; break;
            case ACC_SPMM_ARR_SPARSE_A_TO_B: dev = f.sparse_a_to_b.p; need = (size_t)f.T * f.TW * 4; break;
            case ACC_SPMM_ARR_TC_LOCAL_BIT: dev = f.tc_local_bit.p; need = (size_t)f.T * f.NW * 8; break;
            case ACC_SPMM_ARR_VALUES: dev = f.vals.p; need = (size_t)f.nnz * 2; break;
            default: fail(ACC_SPMM_ERR_INVALID_ARG, "unknown array id");
        }
        if (!host_dst) { *bytes = need; return; }
        if (*bytes < need) fail(ACC_SPMM_ERR_INVALID_ARG, "destination too small");
        *bytes = need;
        if (!need) return;
        if (host) std::memcpy(host_dst, host, need);
        else ACC_HIP(hipMemcpy(host_dst, dev, need, hipMemcpyDeviceToHost));
    });
}

acc_spmm_mtx_t* acc_spmm_mtx_open(const char* path, int32_t value_type) {
    MtxFile* m = nullptr;
    guarded([&] { m = read_matrix_market(path, value_type); });
    return reinterpret_cast<acc_spmm_mtx_t*>(m);
}

int acc_spmm_mtx_shape(const acc_spmm_mtx_t* mtx, int64_t* M, int64_t* K, int64_t* nnz) {
    return guarded([&] {
        if (!mtx) fail(ACC_SPMM_ERR_INVALID_ARG, "null argument");
        matrix_market_shape(reinterpret_cast<const MtxFile*>(mtx), M, K, nnz);
    });
}

int acc_spmm_mtx_csr(const acc_spmm_mtx_t* mtx, int32_t* csr_rowptr, int32_t* csr_colidx, uint16_t* csr_vals) {
    return guarded([&] {
        if (!mtx) fail(ACC_SPMM_ERR_INVALID_ARG, "null argument");
        matrix_market_csr(reinterpret_cast<const MtxFile*>(mtx), csr_rowptr, csr_colidx, csr_vals);
    });
}

void acc_spmm_mtx_close(acc_spmm_mtx_t* mtx) { free_matrix_market(reinterpret_cast<MtxFile*>(mtx)); }

}  // extern "C"
