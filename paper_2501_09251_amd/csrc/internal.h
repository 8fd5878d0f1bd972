// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

#include "acc_spmm.h"

namespace accspmm {

// ---- error plumbing -------------------------------------------------------------------
void set_error(int code, const std::string& msg);
struct Failure {
    int code;
    std::string msg;
};
[[noreturn]] void fail(int code, const std::string& msg);  // throws Failure; caught at the ABI

#define ACC_HIP(expr)                                                                       \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess)                                                               \
            ::accspmm::fail(e_ == hipErrorOutOfMemory ? ACC_SPMM_ERR_OOM : ACC_SPMM_ERR_HIP, \
                            std::string(#expr) + ": " + hipGetErrorString(e_));             \
    } while (0)

// ---- device buffer --------------------------------------------------------------------
template <class T>
struct DevBuf {
    T* p = nullptr;
    size_t n = 0;
    DevBuf() = default;
    DevBuf(const DevBuf&) = delete;
    DevBuf& operator=(const DevBuf&) = delete;
    ~DevBuf() { release(); }
    void alloc(size_t count) {
        release();
        n = count;
        if (count) ACC_HIP(hipMalloc((void**)&p, count * sizeof(T)));
    }
    void release() {
        if (p) (void)hipFree(p);
        p = nullptr;
        n = 0;
    }
    void upload(const T* host, size_t count) {
        alloc(count);
        if (count) ACC_HIP(hipMemcpy(p, host, count * sizeof(T), hipMemcpyHostToDevice));
    }
    void download(T* host) const {
        if (n) ACC_HIP(hipMemcpy(host, p, n * sizeof(T), hipMemcpyDeviceToHost));
    }
    void swap(DevBuf& other) {
        std::swap(p, other.p);
        std::swap(n, other.n);
    }
};

// One unit of runtime work = one wavefront (see acc_spmm_plan_export for the encoding).
struct WorkItem {
    int32_t w_begin, w_end, t_begin, t_end;
};
struct SplitWindow {
    int32_t window, slot_begin, slot_end, pad;
};

// The tile format on the device (paper Section 3.3), for WH x TW tiles.
struct DeviceFormat {
    int32_t WH = 16, TW = 16, NW = 4;  // NW = 64-bit words per tile bitmap
    int64_t M = 0, W = 0, T = 0, nnz = 0, sum_dw = 0;
    DevBuf<int32_t> row_window_offset;  // W+1
    DevBuf<int32_t> tc_offset;          // T+1
    DevBuf<int32_t> sparse_a_to_b;      // T*TW
    DevBuf<uint64_t> tc_local_bit;      // T*NW
    DevBuf<uint16_t> vals;              // nnz (+ padding so that 4 halves past the end are readable)
};

// encode.hip: CSR (device) + perm (device, new->old, M entries) -> DeviceFormat.  entry_of
// (optional) gets, for every packed value position, the index of its CSR entry.
void encode_on_device(int64_t M, int64_t K, int64_t nnz, const int32_t* d_rowptr, const int32_t* d_colidx,
                      const uint16_t* d_vals, const int32_t* d_perm, int32_t WH, int32_t TW, DeviceFormat& out,
                      bool tiles_only, DevBuf<int32_t>* entry_of = nullptr);

// Symmetric adjacency of the pattern graph in (pinned) host memory: vertex i's neighbours,
// ascending, without i itself, are adj[ptr[i] .. ptr[i+1]).
struct HostGraph {
    int64_t M = 0;
    int64_t* ptr = nullptr;
    int32_t* adj = nullptr;
    HostGraph() = default;
    HostGraph(const HostGraph&) = delete;
    HostGraph& operator=(const HostGraph&) = delete;
    ~HostGraph();
};

// The same graph in device memory.
struct DeviceGraph {
    int64_t M = 0, two_m = 0;   // two_m = directed entries = ptr[M]
    DevBuf<int64_t> ptr;        // M+1
    DevBuf<int32_t> adj;        // two_m
};

// graph.hip: the pattern graph of A + A^T (no diagonal) from the device CSR, and its copy to the host.
void build_graph_on_device(int64_t M, int64_t nnz, const int32_t* d_rowptr, const int32_t* d_colidx, DeviceGraph& g);
void copy_graph_to_host(const DeviceGraph& d, HostGraph& g);

// dendrogram.hip: Step I of Algorithm 1 on the GPU (same result as build_dendrogram_host, bit for
// bit).  parent gets M entries (-1 for roots), order the vertices in visiting order (ascending
// degree, ties by id).  work_budget as for build_dendrogram_host.  Returns kDendrogramDone,
// kDendrogramOverBudget (AUTO gives up; outputs unspecified) or kDendrogramUseHost (the device
// form ran out of its memory pools or advances too slowly on this input: the caller runs the host
// form instead).
constexpr int kDendrogramDone = 0, kDendrogramOverBudget = 1, kDendrogramUseHost = 2;
int build_dendrogram_on_device(const DeviceGraph& g, double work_budget, std::vector<int32_t>& parent,
                               std::vector<int32_t>& order, double* work_ratio, int64_t* rounds);

// reorder.cpp: the leaf sequence of a dendrogram given as parent[] plus the visiting order (a
// vertex's children in merge order are its children in visiting order), cut into segments.
void leaf_sequence_from_parents(int64_t M, const std::vector<int32_t>& parent, const std::vector<int32_t>& order,
                                int32_t seg_len, std::vector<int32_t>& seq, std::vector<int64_t>& seg_start);

// reorder.cpp: Step I of Algorithm 1 on the host, and the dendrogram's leaf sequence.
// gptr / gadj: the symmetric adjacency (HostGraph layout).  parent gets M entries (-1 for
// roots); seq the M rows in leaf order; seg_start the first sequence position of every
// segment, terminated by M.  work_budget > 0 limits the dendrogram construction to that many
// edge-record visits per graph entry (vertices + directed edges); when exceeded the function
// returns false and the outputs are unspecified.  *work_ratio (may be null) receives the
// visits per graph entry.
bool build_dendrogram_host(int64_t M, const int64_t* gptr, const int32_t* gadj, int32_t seg_len, double work_budget,
                           std::vector<int32_t>& parent, std::vector<int32_t>& seq, std::vector<int64_t>& seg_start,
                           double* work_ratio);

// ordering.hip: Step II of Algorithm 1 on the GPU.  d_perm gets M entries (new -> old).
void ordering_on_device(int64_t M, int64_t K, int64_t nnz, const int32_t* d_rowptr, const int32_t* d_colidx,
                        const std::vector<int32_t>& seq, const std::vector<int64_t>& seg_start, int32_t seg_len,
                        int32_t max_row_len, DevBuf<int32_t>& d_perm);

// colorder.hip: the plan's column order (d_order: plan column -> input column, d_rank its
// inverse), the relabelling of a column-index array, and the row permutation of a matrix
// (gather: dst row j = src row order[j]; scatter: dst row order[j] = src row j).
void column_order_on_device(int64_t K, int64_t nnz, const int32_t* d_colidx, DevBuf<int32_t>& d_order,
                            DevBuf<int32_t>& d_rank);
void remap_columns_on_device(int64_t nnz, const int32_t* d_colidx, const int32_t* d_rank, int32_t* d_out);
void hot_cold_entries_on_device(int64_t n, int32_t* d_a2b, const int32_t* d_order, int32_t n_hot, int32_t* d_plain);
void launch_permute_rows(const int32_t* d_order, int64_t rows, const void* src, void* dst, int64_t row_bytes, bool scatter,
                         hipStream_t stream);

// schedule.cpp: Section 3.5.
double imbalance_degree(const std::vector<int32_t>& rwo);
void build_schedule(const std::vector<int32_t>& rwo, bool balance, int32_t cap, int32_t WH, int32_t TW,
                    std::vector<WorkItem>& items, std::vector<SplitWindow>& splits, int64_t& n_slots);

struct Plan {
    int device = 0;
    acc_spmm_options opt{};
    acc_spmm_stats stats{};
    DeviceFormat fmt;
    std::vector<int32_t> perm, iperm, parent;  // host copies (perm: new->old)
    DevBuf<int32_t> d_perm_pad;                // W*WH entries, -1 past M
    std::vector<WorkItem> items;
    std::vector<SplitWindow> splits;
    DevBuf<WorkItem> d_items;
    DevBuf<SplitWindow> d_splits;
    int64_t n_slots = 0;
    // partial-sum workspace, grown on demand by execute
    mutable std::mutex workspace_mutex;
    mutable DevBuf<float> workspace;
    mutable int32_t workspace_N = 0;
    // column order (empty when not applied); with B in the caller's order, the first n_hot
    // rows of the order are gathered into b_hot before every execute
    DevBuf<int32_t> d_col_order;
    std::vector<int32_t> col_order, col_rank;
    int32_t n_hot = 0;
    DevBuf<int32_t> a2b_plain;   // SparseAToB with input columns throughout (kept below kDualEntriesMaxK columns)
    mutable DevBuf<uint16_t> b_hot;
    mutable int32_t b_hot_N = 0;
    // optional: CSR entry index of every packed value (for sddmm), and sddmm's results in packed
    // order before they are moved to entry order (allocated by the first sddmm call)
    DevBuf<int32_t> d_entry_of;
    mutable DevBuf<float> sddmm_packed;
    // optional CSR copy for the naive baseline
    DevBuf<int32_t> d_rowptr, d_colidx;
    DevBuf<uint16_t> d_vals;
};

// execute.hip
// tiles_ms non-null: time the kernels with events and wait for them.  narrow_c: C holds 16-bit
// values of the plan's value type instead of fp32.  static_scratch: the call's temporary device
// buffers live in the library's static device array instead of buffers of the plan, and nothing
// is allocated.
void launch_execute(const Plan& plan, const void* B, int32_t N, void* C, hipStream_t stream,
                    float* tiles_ms = nullptr, float* combine_ms = nullptr, float* gather_ms = nullptr,
                    bool narrow_c = false, bool static_scratch = false);
// Looks up, once per device, the address of the static device array behind acc_spmm_execute_static
// on the current device (done when a plan is created, so that the execute call itself has no
// set-up left to do).
void prepare_static_scratch();
void launch_calibration_copy(void* dst, const void* src, size_t bytes, hipStream_t stream);
void launch_calibration_gather(const void* table, int64_t rows, int64_t row_bytes, const int32_t* index, int64_t n_index,
                               void* sink, size_t sink_bytes, void* out, size_t out_bytes, int32_t write_every,
                               int32_t write_rows, hipStream_t stream);
void launch_csr_naive(const Plan& plan, const void* B, int32_t N, void* C, hipStream_t stream);
// sddmm.hip
void launch_update_values(const Plan& plan, const void* csr_vals, hipStream_t stream);
void launch_sddmm(const Plan& plan, const void* X, const void* Y, int32_t N, void* out, int32_t use_values,
                  hipStream_t stream);

// serialize.cpp: a plan to and from a file
void save_plan(const Plan& plan, const char* path);

// mtx.cpp: Matrix Market coordinate file -> host CSR
struct MtxFile;
MtxFile* read_matrix_market(const char* path, int32_t value_type);
void free_matrix_market(MtxFile* m);
void matrix_market_shape(const MtxFile* m, int64_t* M, int64_t* K, int64_t* nnz);
void matrix_market_csr(const MtxFile* m, int32_t* rowptr, int32_t* colidx, uint16_t* vals);

}  // namespace accspmm

struct acc_spmm_mtx_s;  // opaque to callers: an accspmm::MtxFile

struct acc_spmm_plan_s {
    accspmm::Plan plan;
};

namespace accspmm {
acc_spmm_plan_t* load_plan(const char* path);
}
