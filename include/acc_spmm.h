/*
 * acc_spmm.h -- C ABI of the MI355X (gfx950) SpMM library.
 *
 * Computes C = A.B with A sparse M x K (given once as CSR with fp16 values), B dense
 * K x N fp16 and C dense M x N fp32 (problem statement: Acc-SpMM paper, Section 5, first
 * sentence; CSR input: Section 2.2).  The work is split as the paper's overview
 * (Section 3.1) splits it: an offline stage that reorders rows, translates A into the
 * bitmap tile format and balances the load (acc_spmm_plan), and one runtime kernel
 * (acc_spmm_execute).
 *
 * Conventions for every entry point:
 *  - plain C types only; "HOST" / "DEVICE" says where a pointer must live;
 *  - fp16 data is passed as IEEE binary16 bit patterns (uint16_t on the host);
 *  - no entry point throws or aborts: failures return NULL or a negative acc_spmm_status,
 *    and acc_spmm_last_error() gives the message of the calling thread's last failure;
 *  - the library needs a gfx950 device; there is no CPU fallback.
 */
#ifndef ACC_SPMM_H
#define ACC_SPMM_H

#include <stddef.h>
#include <stdint.h>

#define ACC_SPMM_API __attribute__((visibility("default")))

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ACC_SPMM_OK = 0,
    ACC_SPMM_ERR_INVALID_ARG = -1, /* null pointer, negative size, bad option value     */
    ACC_SPMM_ERR_INVALID_CSR = -2, /* rowptr not monotone / rowptr[M] != nnz / column   */
                                   /* out of range / duplicate column inside a row      */
    ACC_SPMM_ERR_UNSUPPORTED = -3, /* N or tile geometry the kernels do not cover       */
    ACC_SPMM_ERR_OOM = -4,         /* host or device allocation failed                  */
    ACC_SPMM_ERR_HIP = -5          /* a HIP runtime call failed (message has the name)  */
} acc_spmm_status;

/* Opaque plan handle, owned by the library; release with acc_spmm_destroy. */
typedef struct acc_spmm_plan_s acc_spmm_plan_t;

/* Values for acc_spmm_options.reorder, .load_balance and .column_order */
enum { ACC_SPMM_OFF = 0, ACC_SPMM_ON = 1, ACC_SPMM_AUTO = 2 };

/* acc_spmm_options.value_type */
enum { ACC_SPMM_FP16 = 0, ACC_SPMM_BF16 = 1 };

/*
 * Plan options.  Zero-initialise, set struct_size = sizeof(acc_spmm_options), then
 * change what you need; a field left 0 takes its default where "0 = default" is stated.
 */
typedef struct {
    int32_t struct_size;
    /* Row reordering (Section 3.2, Algorithm 1).  OFF: identity.  ON: always apply.
     * AUTO (default when struct is NULL): compute it, keep it only if it lowers the number
     * of tiles by at least 1 % (the paper notes in Section 4.3.5 that reordering can lose:
     * it gives up the locality of the input order); AUTO also stops
     * the dendrogram construction, and keeps the identity, once it has visited 8 edge
     * records per graph entry (large uniform meshes, where nothing is gained).
     * Requires M == K; for M != K the dendrogram step is skipped and the order is the
     * identity.  Matrices with nnz >= 2^30 are not reordered: ON returns
     * ACC_SPMM_ERR_UNSUPPORTED for them (before the arrays are read), AUTO keeps the input order. */
    int32_t reorder;
    /* Load balancing (Section 3.5).  OFF: one work item per row window.  ON: always split
     * heavy windows / pack light ones.  AUTO: apply iff IBD (Eq. 3) > ibd_threshold. */
    int32_t load_balance;
    /* Most tiles one work item may hold; heavier windows are split (Section 3.5 uses 32
     * for 8x8x16 tiles on NVIDIA parts).  0 = default: the plan's tiles divided by twice the
     * device's wave slots (12 per compute unit), between 32 and 1024
     * (acc_spmm_stats.max_tiles_per_item reports it). */
    int32_t max_tiles_per_item;
    /* Tile geometry: rows per row window (8, 16, 32 or 64) and condensed columns per tile (8, 16
     * or 32).  0 = default (16,16).  The execute kernel runs (16,16) and (16,32); the latter, on
     * the 32-deep matrix instruction, halves the tiles and measured between 12 % slower and 7 %
     * faster than (16,16) depending on input and N, so no AUTO decision picks it.  A (16,32) plan
     * fetches values as value_fetch = 3, runs pipeline depths 1 and 2 only (deeper requests run
     * as 2), and refuses no_prefetch, lds_staging and acc_spmm_sddmm.  The other geometries,
     * among them the paper's (8,8) (Section 3.3), are accepted for building, exporting and
     * measuring the format only (acc_spmm_plan_stats, acc_spmm_plan_traffic): acc_spmm_execute
     * returns ACC_SPMM_ERR_UNSUPPORTED on such a plan. */
    int32_t window_height;
    int32_t tile_width;
    /* Leaves per segment in the ordering step's candidate search.  0 = default 1024; at
     * most 4096. */
    int32_t segment_length;
    /* IBD threshold for load_balance == AUTO.  0 = default 8 (Section 3.5). */
    float ibd_threshold;
    /* Keep a device copy of the input CSR so that acc_spmm_execute_csr_naive works. */
    int32_t keep_csr;
    /* Ablation switch: 0 = default (software-pipelined loads, Section 3.4), 1 = issue each
     * tile's loads only when the tile is computed. */
    int32_t no_prefetch;
    /* Cache policy of the C stores (Section 3.4 writes C through, uncached): 0 = default,
     * ordinary stores, which measure about 5 % faster on MI355X; 1 = streaming
     * (non-temporal) stores, the counterpart of the paper's write-through policy. */
    int32_t streaming_stores;
    /* Tiles of B rows kept in flight per wavefront while one tile is multiplied (1..3).
     * 0 = default: 1 for plans with fewer than 64 tiles per work item; else 3 where a wavefront
     * takes one 128-feature slab and 2 otherwise.  Ignored when
     * no_prefetch is set. */
    int32_t pipeline_depth;
    /* How a tile's packed values reach the lanes of the wavefront: 1 = every lane loads its
     * own up-to-four values one by one; 2 = the wavefront loads the tile's values once and the
     * lanes exchange them across registers; 3 = every lane loads the twelve bytes around its
     * (consecutive) values at once; 0 = default, by the lane width the call uses (a width N that
     * is not a multiple of 8 counts as the narrower class):
     *   N <= 32: 3; but 1 if the plan has 64 tiles or more per work item and its windows share
     *     almost no columns (at least 0.95 gathered rows of B per entry);
     *   32 < N <= 64: 2 when the plan has at least 24 entries per tile on average or at least
     *     16384 tiles, else 1;
     *   N > 64: 3 when the plan has at least 24 entries per tile on average or fewer than 64
     *     tiles per work item, else 1. */
    int32_t value_fetch;
    /* The 16-bit floating-point type of csr_vals and of B: ACC_SPMM_FP16 (0, default) = IEEE
     * binary16, ACC_SPMM_BF16 (1) = bfloat16.  C is fp32 and products are accumulated in fp32
     * either way. */
    int32_t value_type;
    /* Column order of A = row order of B inside the plan (the paper names column reordering
     * with the matching row reordering of B as the step after row reordering; Section 4.3.1
     * and the conclusion).  ON: columns are grouped by floor(log2(entries in the column)),
     * classes descending, input ids ascending inside a class, unused columns last, so the
     * rows of B that many windows gather sit together whatever labels the input gave them.
     * AUTO: ON when K >= 2^20 (B then exceeds the memory-side cache at usual N) and the
     * labels of the most used columns are concentrated on few residues modulo 16, 256 or
     * 4096 (acc_spmm_stats.hub_label_skew >= 4), which is when gathering their rows of B
     * collides in the memory system; else OFF. */
    int32_t column_order;
    /* 0: B is given in the caller's row order; when the plan has a column order, every
     *    execute first gathers the rows of B for the first min(K/16, 2^17) columns of that
     *    order (the most used ones) into a buffer of the plan and reads the other rows of B
     *    in place (plans with K < 2^22 read all of B in place when N <= 64, where the gathered
     *    copy does not pay).
     * 1: B is given in the plan's order already (B_plan[j] = B[col_order[j]], see
     *    acc_spmm_permute_rows and ACC_SPMM_ARR_COL_ORDER); execute reads it in place.
     * C is in the caller's row order in both cases. */
    int32_t operand_order;
    /* 1: keep, for every packed value, the index of its CSR entry (4 bytes per entry), which
     * acc_spmm_sddmm needs. */
    int32_t keep_entry_map;
    /* Step I of the reordering (Algorithm 1, dendrogram construction) runs on the GPU, in rounds that
     * reproduce the sequential result; 1 runs its sequential host form instead (same result; for
     * comparison).  The library switches to the host form by itself when the input does not suit the
     * device form (acc_spmm_stats.dendrogram_on_device tells which one ran). */
    int32_t dendrogram_on_host;
    /* Comparison switch: 1 stages the gathered rows of B through a double buffer in LDS, as the
     * paper's Algorithm 2 does (global memory -> LDS for tile k+1 while tile k is multiplied), instead
     * of the register ring, which measured as fast or faster everywhere and is the default.  Same
     * result bit for bit.  fp16 plans, N = 32, 64, 128 or 384; other calls return
     * ACC_SPMM_ERR_UNSUPPORTED. */
    int32_t lds_staging;
    /* Feature slabs (16 times the features per lane, 128 features at N >= 128) that one wavefront
     * accumulates: 2 halves the reads of A and of the index words, 1 puts twice the wavefronts on
     * the rows of B.  0 = default: 1 when the plan has fewer than 24 entries per tile on average and
     * the call gathers the most used rows of B (a column order with B in the caller's order), else
     * 2 where N spans an even number of slabs or more than three.  1 and 2 force it where the
     * width allows (2 needs at least two slabs). */
    int32_t slabs_per_wave;
} acc_spmm_options;

/* What a plan holds; filled by acc_spmm_plan_stats. */
typedef struct {
    int64_t M, K, nnz;
    int32_t window_height, tile_width;
    int64_t num_windows;        /* W = ceil(M / window_height)                               */
    int64_t num_tiles;          /* T = NumTcBlock                                            */
    int64_t sum_distinct_cols;  /* sum over windows of distinct column indices (B rows read) */
    int64_t num_tiles_identity; /* T with the identity order (== num_tiles if reorder off)   */
    int64_t num_items;          /* work items (one wavefront each) in the schedule           */
    int64_t num_split_windows;  /* windows whose tiles are spread over several items         */
    int64_t num_partial_slots;  /* partial C tiles (window_height x N fp32) in the workspace */
    int32_t max_tiles_per_item;
    int32_t reorder_applied, load_balance_applied;
    double ibd;                 /* Eq. 3 on the final tile counts                            */
    double mean_nnz_per_tile;   /* MeanNNZTC (Section 4.3.1) = nnz / T                       */
    int64_t index_bytes;        /* RowWindowOffset + TCOffset + SparseAToB + TCLocalBit      */
    int64_t schedule_bytes;     /* work items + permutation                                  */
    double reorder_work_ratio;  /* dendrogram edge-record visits per graph entry (0 if not run)  */
    double t_validate_s, t_reorder_s, t_encode_s, t_schedule_s, t_total_s;
    double t_graph_s, t_dendrogram_s, t_ordering_s; /* parts of t_reorder_s (the rest: tile counting) */
    int32_t column_order_applied;
    int32_t num_hot_columns;    /* rows of B gathered per execute (operand_order 0 with a column order) */
    double hub_label_skew;      /* most loaded residue class of the most used columns' labels,  */
                                /* relative to an even spread (0 if not computed: column_order */
                                /* OFF or K < 65536)                                           */
    double t_column_order_s;
    int32_t dendrogram_on_device; /* 1: Step I of the reordering ran in its device form          */
    int32_t pad_;
    int64_t dendrogram_rounds;    /* rounds of the device form, those before a handover to the  */
                                  /* host form included (0 if the host form was asked for)      */
} acc_spmm_stats;

/* Arrays acc_spmm_plan_export can copy out (element type, element count). */
typedef enum {
    ACC_SPMM_ARR_PERM = 0,              /* int32  M          new row -> input row           */
    ACC_SPMM_ARR_IPERM = 1,             /* int32  M          input row -> new row           */
    ACC_SPMM_ARR_ROW_WINDOW_OFFSET = 2, /* int32  W+1                                       */
    ACC_SPMM_ARR_TC_OFFSET = 3,         /* int32  T+1                                       */
    ACC_SPMM_ARR_SPARSE_A_TO_B = 4,     /* int32  T*tile_width; input columns, or, with a   */
                                        /*        column order: plan columns (operand_order */
                                        /*        1), or ~p for plan column p < num_hot_    */
                                        /*        columns and the input column otherwise    */
                                        /*        (operand_order 0)                         */
    ACC_SPMM_ARR_TC_LOCAL_BIT = 5,      /* uint64 T*ceil(window_height*tile_width/64)       */
    ACC_SPMM_ARR_VALUES = 6,            /* uint16 nnz        fp16 bits in tile order        */
    ACC_SPMM_ARR_WORK_ITEMS = 7,        /* int32  4*num_items, see acc_spmm_plan_export     */
    ACC_SPMM_ARR_DENDROGRAM_PARENT = 8, /* int32  M          -1 for roots; empty if reorder */
                                        /*                   was off                        */
    ACC_SPMM_ARR_COL_ORDER = 9,         /* int32  K          plan column -> input column    */
    ACC_SPMM_ARR_COL_RANK = 10          /* int32  K          input column -> plan column    */
                                        /*                   (both empty without a column   */
                                        /*                   order)                         */
} acc_spmm_array;

/*
 * Build a plan with default options (reorder AUTO, load balance AUTO, 16x16 tiles).
 *   M, K, nnz    shape of A and number of stored entries; 0 <= M, K < 2^31, 0 <= nnz < 2^31
 *   csr_rowptr   HOST int32[M+1], rowptr[0] == 0, non-decreasing, rowptr[M] == nnz
 *   csr_colidx   HOST int32[nnz], each in [0,K); order inside a row is free, duplicates
 *                inside a row are an error
 *   csr_vals     HOST uint16[nnz], fp16 bit patterns (a stored 0.0 stays a stored entry)
 * The arrays are only read during the call.  Returns NULL on failure.
 * The plan lives on the HIP device that is current when this is called.
 */
ACC_SPMM_API acc_spmm_plan_t* acc_spmm_plan(int64_t M, int64_t K, int64_t nnz, const int32_t* csr_rowptr,
                               const int32_t* csr_colidx, const uint16_t* csr_vals);

/* Same, with options (NULL = defaults). */
ACC_SPMM_API acc_spmm_plan_t* acc_spmm_plan_ex(int64_t M, int64_t K, int64_t nnz, const int32_t* csr_rowptr,
                                  const int32_t* csr_colidx, const uint16_t* csr_vals,
                                  const acc_spmm_options* options);

/* Same as acc_spmm_plan_ex for CSR arrays that live in DEVICE memory (of the current device):
 * they are copied to the host first, since the plan validates and reorders there. */
ACC_SPMM_API acc_spmm_plan_t* acc_spmm_plan_device(int64_t M, int64_t K, int64_t nnz, const int32_t* csr_rowptr,
                                                   const int32_t* csr_colidx, const uint16_t* csr_vals,
                                                   const acc_spmm_options* options);

/*
 * Enqueue C = A.B on `stream` (Algorithm 2's runtime kernel; Section 3.5's split row
 * windows are combined by a second small kernel on the same stream).
 *   B       DEVICE fp16, row-major K x N, leading dimension N, 16-byte aligned
 *   N       1 .. 65536.  A lane of the kernel handles the largest power of two of features,
 *           up to 8, that divides N, so multiples of 8 run at full speed (each lane reads 16
 *           bytes of a B row at once), other even N slower, odd N slowest; 16, 32, 64 and
 *           multiples of 128 leave no lane idle
 *   C       DEVICE fp32, row-major M x N, leading dimension N, 16-byte aligned; every
 *           element is overwritten (rows without entries become 0); rows are in the
 *           caller's original order whatever the plan's internal reordering
 *   stream  hipStream_t, NULL = the default stream
 * Returns without waiting for the GPU.  Calls on one plan must not overlap in time on
 * different streams when the plan has split windows or gathers rows of B (they share the
 * plan's partial-sum workspace and its buffer for the gathered rows, which the first call
 * with a larger N (re)allocates).  A call that would have to (re)allocate while `stream` is
 * being captured into a HIP graph allocates nothing and returns ACC_SPMM_ERR_INVALID_ARG:
 * make one call at that N before the capture, or use acc_spmm_execute_static.
 */
ACC_SPMM_API int acc_spmm_execute(const acc_spmm_plan_t* plan, const void* B, int32_t N, void* C, void* stream);

/*
 * acc_spmm_execute with C in 16 bits: C is DEVICE row-major M x N in the plan's value type
 * (IEEE half or bfloat16), each element the fp32 result rounded to nearest even.  The
 * accumulation is in fp32 as in acc_spmm_execute (the partial sums of split windows too); only
 * the final store is narrow, which halves the bytes written.  Not an operation of the paper
 * (its C is fp32): for layers that would round C to 16 bits anyway.  Same arguments, alignment
 * (C 16-byte aligned), errors and stream behaviour as acc_spmm_execute.
 */
ACC_SPMM_API int acc_spmm_execute_c16(const acc_spmm_plan_t* plan, const void* B, int32_t N, void* C, void* stream);

/*
 * acc_spmm_execute for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, result (bit for bit) and
 * kernels as acc_spmm_execute, but the call's two temporary device buffers (the partial tiles of
 * split row windows, num_partial_slots x 16 x N fp32, and, when the plan gathers rows of B, the
 * num_hot_columns x N gathered rows) are carved out of one array of
 * ACC_SPMM_STATIC_SCRATCH_BYTES that the library holds in device memory of every GPU it runs on
 * from load time until the process ends.  It calls no hipMalloc / hipFree and no allocating
 * library routine.  A plan whose two buffers at this N (the first rounded up to 256 bytes) exceed
 * that size is refused with ACC_SPMM_ERR_UNSUPPORTED and a message that gives both sizes;
 * acc_spmm_execute serves it.  Nothing in the array has to be cleared between calls: every
 * element a call reads was written earlier in the same call.  All calls on one GPU, from any plan
 * and any stream, share the array, so calls that overlap in time on one GPU race: order them on
 * one stream, or with events.
 */
#define ACC_SPMM_STATIC_SCRATCH_BYTES (64u << 20)
ACC_SPMM_API int acc_spmm_execute_static(const acc_spmm_plan_t* plan, const void* B, int32_t N, void* C, void* stream);

/*
 * acc_spmm_execute with per-kernel timing, for benchmarks: records HIP events on `stream`
 * around the gather of B (if the plan does one), the tile kernel and the split-window
 * combine kernel, waits for them, and returns the durations in milliseconds (gather_ms and
 * combine_ms, which may be NULL, are 0 when the plan runs no such kernel).  Same contract
 * as acc_spmm_execute otherwise, but it blocks the calling thread.
 */
ACC_SPMM_API int acc_spmm_execute_timed(const acc_spmm_plan_t* plan, const void* B, int32_t N, void* C,
                                        void* stream, float* tiles_ms, float* combine_ms, float* gather_ms);

/*
 * Sampled dense-dense product on the plan's sparsity pattern (the companion of SpMM in graph
 * neural network layers; not an operation of the paper, whose Section 5 names use from GNN
 * frameworks as the goal): for every stored entry p = (i, j) of A
 *     out[p] = sum over f < N of X[i][f] * Y[j][f]        (times A's value at p if use_values)
 * on the matrix cores, fp32 accumulation.  Needs a plan built with keep_entry_map = 1.
 *   X    DEVICE 16-bit floats (the plan's value_type), row-major M x N, rows in the caller's order
 *   Y    DEVICE, row-major K x N, rows as acc_spmm_execute takes B (operand_order; in the
 *        caller's order the most used rows are gathered first, as for B)
 *   N    32, 64, 96, 128, or a multiple of 128 up to 4096
 *   out  DEVICE fp32[nnz], entry p in row-major order with ascending columns inside a row
 *        (the order of csr_colidx when its rows are sorted)
 * X and Y 16-byte aligned.  Enqueues two kernels on `stream` and returns; the first call
 * allocates a buffer of nnz floats in the plan, which calls that overlap in time would share.
 */
ACC_SPMM_API int acc_spmm_sddmm(const acc_spmm_plan_t* plan, const void* X, const void* Y, int32_t N, void* out,
                                int32_t use_values, void* stream);

/*
 * Replace the values of A, keeping its pattern (and with it the whole plan): layers that
 * recompute edge weights every step, for instance from acc_spmm_sddmm's output, re-use one plan.
 *   csr_vals  DEVICE uint16[nnz], bit patterns of the plan's value_type, entry p in row-major
 *             order with ascending columns inside a row (acc_spmm_sddmm's output order)
 * Needs a plan built with keep_entry_map = 1.  Enqueues on `stream`; later executes on that
 * stream see the new values.  The copy kept for acc_spmm_execute_csr_naive is not updated.
 */
ACC_SPMM_API int acc_spmm_update_values(acc_spmm_plan_t* plan, const void* csr_vals, void* stream);

/*
 * Reorder the rows of a K-row DEVICE matrix between the caller's order and the plan's
 * column order (for callers that keep B in the plan's order, options.operand_order = 1).
 *   row_bytes  bytes per row, a multiple of 2
 *   to_caller  0: dst[j] = src[col_order[j]] (caller's order -> plan's order)
 *              1: dst[col_order[j]] = src[j] (plan's order -> caller's order)
 * src and dst must not overlap.  Without a column order in the plan this is a plain copy.
 */
ACC_SPMM_API int acc_spmm_permute_rows(const acc_spmm_plan_t* plan, const void* src, void* dst, int64_t row_bytes,
                                       int32_t to_caller, void* stream);

/*
 * Baseline for comparisons: one wavefront per CSR row, fp32 FMA, no tiles, no matrix
 * cores.  Needs a plan built with keep_csr = 1.  Same B / N / C / stream contract, any N >= 1.
 */
ACC_SPMM_API int acc_spmm_execute_csr_naive(const acc_spmm_plan_t* plan, const void* B, int32_t N, void* C, void* stream);

/* Releases a plan and its device memory (utility call, no passage of the paper).  NULL is
 * allowed.  The caller must have waited for every execute that uses the plan. */
ACC_SPMM_API void acc_spmm_destroy(acc_spmm_plan_t* plan);

/*
 * A plan on disk (the paper amortises the preprocessing over iterative use, Section 4.3.2;
 * this carries it across processes).  acc_spmm_plan_save writes everything execute, sddmm,
 * update_values, the comparison kernel and plan_export need to `path`; acc_spmm_plan_load
 * reads such a file into a new plan on the current HIP device (NULL on failure, reason in
 * acc_spmm_last_error).  The file is only meant for the library version and machine type
 * that wrote it: another version is refused with ACC_SPMM_ERR_UNSUPPORTED.  The file ends
 * in a checksum; one that was cut short or whose bytes changed is refused with
 * ACC_SPMM_ERR_INVALID_ARG and no kernel ever sees its contents.
 */
ACC_SPMM_API int acc_spmm_plan_save(const acc_spmm_plan_t* plan, const char* path);
ACC_SPMM_API acc_spmm_plan_t* acc_spmm_plan_load(const char* path);

/* Message of the calling thread's last failure; returns its status code (0 if none).
 * buf may be NULL.  (Utility call, no passage of the paper.) */
ACC_SPMM_API int acc_spmm_last_error(char* buf, size_t len);

ACC_SPMM_API int acc_spmm_plan_stats(const acc_spmm_plan_t* plan, acc_spmm_stats* out);

/*
 * Bytes the method must move for one execute at width N, counted from the plan
 * (A values once, A indices once, each window's distinct B rows once, C once), and the
 * dense flops the matrix cores are issued.  Any output pointer may be NULL.
 */
ACC_SPMM_API int acc_spmm_plan_traffic(const acc_spmm_plan_t* plan, int32_t N, int64_t* a_bytes, int64_t* b_bytes,
                          int64_t* c_bytes, int64_t* mfma_flops);

/*
 * Copy one of the plan's arrays to HOST memory: the four index arrays and the packed values of
 * the tile format (Section 3.3), the row permutation and the dendrogram (Section 3.2, Algorithm
 * 1), the work items (Section 3.5) and the column order: what the parity tests compare.
 * Pass host_dst == NULL to get the size in bytes through *bytes; otherwise *bytes must be at
 * least that size.
 * Work items are 4 x int32 {w_begin, w_end, t_begin, t_end}:
 *   w_end >  w_begin : the item owns windows [w_begin, w_end) completely
 *                      (t_begin, t_end are their first and one-past-last tile);
 *   w_end <  0       : the item owns tiles [t_begin, t_end) of window w_begin and writes
 *                      partial slot (-w_end - 1).
 */
ACC_SPMM_API int acc_spmm_plan_export(const acc_spmm_plan_t* plan, int which, void* host_dst, size_t* bytes);

/*
 * Matrix Market files (the format of the SuiteSparse and graph collections the paper
 * evaluates on, Section 4.1) -> the HOST CSR arrays acc_spmm_plan takes.  Host code only; no
 * GPU is needed.
 *   acc_spmm_mtx_open   parses `path` ("matrix coordinate", field real / integer / pattern,
 *                       symmetry general / symmetric / skew-symmetric; the stored triangle
 *                       of a symmetric file is mirrored, pattern entries get the value 1,
 *                       entries given twice are summed) and converts the values to
 *                       value_type (ACC_SPMM_FP16 or ACC_SPMM_BF16, round to nearest even;
 *                       magnitudes beyond the type's range become infinity).  Returns NULL
 *                       on failure (acc_spmm_last_error has the reason).
 *   acc_spmm_mtx_shape  M, K and the number of stored entries (any pointer may be NULL)
 *   acc_spmm_mtx_csr    copies out rowptr[M+1], colidx[nnz] (ascending inside a row) and
 *                       vals[nnz]; a NULL array is skipped
 *   acc_spmm_mtx_close  releases the handle
 */
typedef struct acc_spmm_mtx_s acc_spmm_mtx_t;
ACC_SPMM_API acc_spmm_mtx_t* acc_spmm_mtx_open(const char* path, int32_t value_type);
ACC_SPMM_API int acc_spmm_mtx_shape(const acc_spmm_mtx_t* mtx, int64_t* M, int64_t* K, int64_t* nnz);
ACC_SPMM_API int acc_spmm_mtx_csr(const acc_spmm_mtx_t* mtx, int32_t* csr_rowptr, int32_t* csr_colidx, uint16_t* csr_vals);
ACC_SPMM_API void acc_spmm_mtx_close(acc_spmm_mtx_t* mtx);

/*
 * Measurement aid: a plain streaming copy kernel (16 bytes per lane, grid-stride) that
 * reads `bytes` from src and writes them to dst (both DEVICE, 16-byte aligned, bytes a
 * multiple of 16).  Hardware counters read for it calibrate the counters read for the
 * SpMM kernels.
 */
ACC_SPMM_API int acc_spmm_calibration_copy(void* dst, const void* src, size_t bytes, void* stream);

/*
 * Measurement aid: the memory pattern of the tile kernel's gather of B rows and nothing else
 * (Section 3.4 names this gather as where the time goes).  For every 16 entries of `index` (one
 * "tile") a wavefront reads those 16 rows of `table`, 16 bytes per lane and 256 contiguous bytes
 * per 16 lanes, four tiles in flight; the data is folded into `sink`.  With write_rows > 0 every
 * wavefront also streams write_rows rows of 2 * row_bytes (the fp32 image of a row) to `out` after
 * every write_every tiles, as the tile kernel writes the rows of a window of C after its tiles.
 *   table        DEVICE, rows x row_bytes, row_bytes a multiple of 16
 *   index        DEVICE int32[n_index], every entry in [0, rows) (not checked: it lives on the
 *                device), n_index a multiple of 16
 *   sink         DEVICE, at least 16 MiB, overwritten
 *   out          DEVICE, needed when write_rows > 0: at least W * ceil(ceil(T / W) / write_every)
 *                * write_rows * 2 * row_bytes bytes for T = n_index / 16 tiles and
 *                W = 4 * min(ceil(T / 4), 4096) wavefronts (the call checks out_bytes against
 *                this and says how many are needed); write_every a multiple of 4
 * All pointers 16-byte aligned.  Timed by the caller (events on `stream`): the rate of this call
 * is the ceiling the tile kernel's gather can reach on the machine at hand.
 */
ACC_SPMM_API int acc_spmm_calibration_gather(const void* table, int64_t rows, int64_t row_bytes, const int32_t* index,
                                             int64_t n_index, void* sink, size_t sink_bytes, void* out, size_t out_bytes,
                                             int32_t write_every, int32_t write_rows, void* stream);

/*
 * The two host-side stages of acc_spmm_plan, callable on their own (no GPU needed).
 *
 * acc_spmm_dendrogram_host: Step I of the row reordering of Section 3.2 (Algorithm 1,
 * dendrogram construction) and the leaf sequence Step II starts from.  Input (HOST): the
 * pattern graph as symmetric adjacency, graph_rowptr int64[M+1] and graph_adj int32 with
 * vertex i's neighbours in graph_adj[graph_rowptr[i] .. graph_rowptr[i+1]), ascending,
 * without i itself (inside acc_spmm_plan the GPU builds this from A + A^T).  segment_length
 * 0 = default.  Outputs (HOST): parent int32[M] (community each vertex was merged into, -1
 * for roots); leaf_sequence int32[M] (may be NULL: the rows in depth-first leaf order);
 * segment_start int32[M+1] (may be NULL: first sequence position of every segment, followed
 * by M).  *work_ratio (may be NULL) receives the edge-record visits per graph entry
 * (vertices + directed edges), the quantity acc_spmm_plan's AUTO mode limits.
 * Returns the number of segments, or a negative acc_spmm_status.
 *
 * acc_spmm_schedule_host: Section 3.5 for 16x16 tiles.  row_window_offset is HOST
 * int32[W+1].  load_balance / max_tiles_per_item / ibd_threshold as in acc_spmm_options,
 * except that max_tiles_per_item 0 means 256 here (there is no device to size it by).
 * *ibd_out receives Eq. 3 (may be NULL).  Work items (4 x int32 each, encoding as for
 * acc_spmm_plan_export) are written to `items` if it is not NULL; items_capacity is its
 * capacity in items.  Returns the number of work items, or a negative acc_spmm_status.
 */
ACC_SPMM_API int64_t acc_spmm_dendrogram_host(int64_t M, const int64_t* graph_rowptr, const int32_t* graph_adj,
                                              int32_t segment_length, int32_t* parent, int32_t* leaf_sequence,
                                              int32_t* segment_start, double* work_ratio);

ACC_SPMM_API int64_t acc_spmm_schedule_host(int64_t W, const int32_t* row_window_offset, int32_t load_balance,
                               int32_t max_tiles_per_item, float ibd_threshold, double* ibd_out,
                               int32_t* items, int64_t items_capacity, int64_t* num_partial_slots);

#ifdef __cplusplus
}
#endif
#endif /* ACC_SPMM_H */
