// Sampled dense-dense product on the plan's tile format: for every stored entry (i, j) of A,
//     out = sum_f X[i][f] * Y[j][f]        (optionally times the entry's value),
// the companion of SpMM in graph neural network layers (the paper's stated goal is use from
// GNN frameworks, Section 5; the operation itself is not in the paper).  The tile format
// makes it a dense contraction: for a 16x16 tile, rows of X for the window's 16 rows against
// the 16 gathered rows of Y, over the N features, on v_mfma_f32_16x16x16; the bitmap then
// says which of the 256 results are entries, and the popcount rank says where they go.
//
// One wavefront per work item of the SpMM schedule (tiles are independent here, so split
// windows need no combining).  Lane (g = lane/16, c = lane%16) holds, of row c of the
// window (A operand) and of gathered row c of the tile (B operand), the features
// [32v + 8g, 32v + 8g + 8) for v = 0 .. N/32-1: one 16-byte load each, and the four lane
// groups together read 64 contiguous bytes of a row.  The contraction index may be visited
// in any order as long as both operands agree, so no transpose is needed.  A wave keeps its
// window's rows of X in registers and double-buffers the rows of Y (the column ids of tile
// t+2 are requested before the rows of tile t+1, so that waiting for ids never drains data).
// The tile kernel writes its results in the plan's packed value order and loads nothing that
// depends on them; a second, streaming kernel moves them to the caller's entry order and
// applies the entries' values.  (With the map lookup inside the tile kernel, every tile waited
// on a load issued after the prefetch of the next tile's rows, which drained the pipeline.)
#include <algorithm>
#include <mutex>
#include <type_traits>

#include "execute.h"

namespace accspmm {
namespace {

typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));

// NV = 16-byte loads per lane and row in one pass over the features (N = 32 * NV * passes).
// PASSES > 0: that many passes, the window's rows of X stay in registers and the rows of Y are
// double-buffered pass by pass.  PASSES == 0: any number of passes (`passes`), X and Y re-read
// per tile and pass, no prefetch (very wide rows).
// HOT: SparseAToB entries e < 0 name row ~e of Y_hot, the plan's gathered copy of the most used
// rows of Y (the plan has a column order and Y comes in the caller's order); e >= 0 are rows of Y.
template <int NV, int PASSES, bool BF16, bool HOT>
__global__ __launch_bounds__(kWavesPerBlock * 64) void sddmm_tiles_kernel(
    const int32_t* __restrict__ rwo, const int32_t* __restrict__ tco, const int32_t* __restrict__ a2b,
    const uint64_t* __restrict__ bits, const int32_t* __restrict__ perm_pad, const WorkItem* __restrict__ items,
    const uint16_t* __restrict__ X, const uint16_t* __restrict__ Y, const uint16_t* __restrict__ Y_hot,
    float* __restrict__ packed_out, int32_t n_items, int32_t n_blocks, int32_t N, int32_t passes) {
    const int lane = threadIdx.x & 63;
    const int g = lane >> 4, c = lane & 15;
    const int per_xcd = (n_blocks + 7) >> 3;
    const int lblock = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (lblock >= n_blocks) return;
    const int item_id = __builtin_amdgcn_readfirstlane(lblock * kWavesPerBlock + (int)(threadIdx.x >> 6));
    if (item_id >= n_items) return;
    const WorkItem it = items[item_id];
    const int tb = __builtin_amdgcn_readfirstlane(it.t_begin);
    const int te = __builtin_amdgcn_readfirstlane(it.t_end);
    if (tb >= te) return;
    int w = __builtin_amdgcn_readfirstlane(it.w_begin);
    while (rwo[w + 1] <= tb) ++w;  // the window of the first tile (whole-window items may start with empty windows)
    int wend = rwo[w + 1];

    // a row's address is one 32x32+64-bit multiply-add on the lane's byte address in row 0 of the matrix
    const uint32_t row_bytes = (uint32_t)N * 2u;
    const uint64_t x_base = reinterpret_cast<uint64_t>(X) + (uint64_t)g * 16;
    const uint64_t y_base = reinterpret_cast<uint64_t>(Y) + (uint64_t)g * 16;
    const uint64_t y_hot_base = reinterpret_cast<uint64_t>(Y_hot) + (uint64_t)g * 16;
    auto load_row = [&](uint64_t base, int32_t row, int pass, uintx4 (&dst)[NV]) __attribute__((always_inline)) {
        // named as global memory: a pointer made from an integer would be a generic one, and generic
        // loads also count on the wait counter of the scalar loads
        const uint64_t a = (uint64_t)(uint32_t)row * (uint64_t)row_bytes + base + (uint64_t)(pass * (NV * 64));
#pragma unroll
        for (int v = 0; v < NV; ++v)
            dst[v] = *reinterpret_cast<const __attribute__((address_space(1))) uintx4*>(a + (uint64_t)(v * 64));
    };
    auto load_y = [&](int32_t e, int pass, uintx4 (&dst)[NV]) __attribute__((always_inline)) {
        if constexpr (HOT) {
            const bool hot = e < 0;
            load_row(hot ? y_hot_base : y_base, hot ? ~e : e, pass, dst);
        } else {
            load_row(y_base, e, pass, dst);
        }
    };
    auto contract = [&](const uintx4 (&x)[NV], const uintx4 (&y)[NV], floatx4& acc) __attribute__((always_inline)) {
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uintx2 a{h ? x[v].z : x[v].x, h ? x[v].w : x[v].y};
                const uintx2 b{h ? y[v].z : y[v].x, h ? y[v].w : y[v].y};
                if constexpr (BF16)
                    acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(shortx4, a),
                                                                    __builtin_bit_cast(shortx4, b), acc, 0, 0, 0);
                else
                    acc = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(half4, a), __builtin_bit_cast(half4, b),
                                                                acc, 0, 0, 0);
            }
    };
    // the index words of a tile that are needed after its contraction: bitmap and TCOffset
    // (wave-uniform); requested a tile ahead together with the column ids
    struct TileWords {
        uint64_t b0, b1, b2, b3;
        int32_t tco;
    };
    auto load_words = [&](int t) __attribute__((always_inline)) {
        const uint64_t* bm = bits + (size_t)t * 4;
        return TileWords{bm[0], bm[1], bm[2], bm[3], tco[t]};
    };
    // results of a tile: lane (g, c) holds rows 4g..4g+3 of column c; bit (4g+r)*16 + c lies in
    // word g of the bitmap at position 16r + c
    auto emit = [&](const TileWords& tw, const floatx4& acc) __attribute__((always_inline)) {
        const int c0 = __builtin_popcountll(tw.b0), c1 = __builtin_popcountll(tw.b1), c2 = __builtin_popcountll(tw.b2);
        const uint64_t word = g == 0 ? tw.b0 : (g == 1 ? tw.b1 : (g == 2 ? tw.b2 : tw.b3));
        const int before = tw.tco + (g >= 1 ? c0 : 0) + (g >= 2 ? c1 : 0) + (g >= 3 ? c2 : 0);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int pos = 16 * r + c;
            if ((word >> pos) & 1ull) packed_out[before + __builtin_popcountll(word & ((1ull << pos) - 1ull))] = acc[r];
        }
    };

    if constexpr (PASSES == 1) {
        uintx4 x[NV], y0[NV], y1[NV];
        auto load_window = [&]() __attribute__((always_inline)) {
            const int32_t row = perm_pad[(size_t)w * 16 + c];
#pragma unroll
            for (int v = 0; v < NV; ++v) x[v] = uintx4{0u, 0u, 0u, 0u};
            if (row >= 0) load_row(x_base, row, 0, x);
        };
        load_window();
        // column ids are requested one tile further ahead than the rows they address
        int32_t col_after = a2b[(size_t)(tb + 1 < te ? tb + 1 : tb) * 16 + c];
        load_y(a2b[(size_t)tb * 16 + c], 0, y0);
        TileWords words_next = load_words(tb);
        auto tile_step = [&](int t, const uintx4 (&y_cur)[NV], uintx4 (&y_next)[NV]) __attribute__((always_inline)) {
            const TileWords words = words_next;
            words_next = load_words(t + 1 < te ? t + 1 : t);
            const int32_t col_ahead = a2b[(size_t)(t + 2 < te ? t + 2 : te - 1) * 16 + c];
            if (t + 1 < te) load_y(col_after, 0, y_next);
            col_after = col_ahead;
            if (t == wend) {  // the previous tile closed its window: move to the window of tile t
                do { ++w; wend = rwo[w + 1]; } while (wend <= t);
                load_window();
            }
            floatx4 acc{0.f, 0.f, 0.f, 0.f};
            contract(x, y_cur, acc);
            emit(words, acc);
        };
        for (int t = tb; t < te; t += 2) {
            tile_step(t, y0, y1);
            if (t + 1 < te) tile_step(t + 1, y1, y0);
        }
    } else if constexpr (PASSES > 1) {
        uintx4 x[PASSES][NV], y0[NV], y1[NV];
        auto load_window = [&]() __attribute__((always_inline)) {
            const int32_t row = perm_pad[(size_t)w * 16 + c];
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
#pragma unroll
                for (int v = 0; v < NV; ++v) x[p][v] = uintx4{0u, 0u, 0u, 0u};
                if (row >= 0) load_row(x_base, row, p, x[p]);
            }
        };
        load_window();
        // column ids are requested a tile before the rows they address are
        int32_t col_cur = a2b[(size_t)tb * 16 + c];
        int32_t col_next = a2b[(size_t)(tb + 1 < te ? tb + 1 : tb) * 16 + c];
        load_y(col_cur, 0, y0);
        TileWords words_next = load_words(tb);
        // One tile: its passes are unrolled, the two buffers alternating pass by pass; START says
        // which buffer holds the tile's first pass (it alternates tile by tile when PASSES is odd).
        auto tile_step = [&](int t, auto start_tag) __attribute__((always_inline)) {
            constexpr int START = decltype(start_tag)::value;
            const TileWords words = words_next;
            words_next = load_words(t + 1 < te ? t + 1 : t);
            const int32_t col_ahead = a2b[(size_t)(t + 2 < te ? t + 2 : te - 1) * 16 + c];
            if (t == wend) {  // the previous tile closed its window: move to the window of tile t
                do { ++w; wend = rwo[w + 1]; } while (wend <= t);
                load_window();
            }
            floatx4 acc{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                const bool last_pass = p == PASSES - 1;
                if (((START + p) & 1) == 0) {
                    if (!last_pass) load_y(col_cur, p + 1, y1);
                    else if (t + 1 < te) load_y(col_next, 0, y1);
                    contract(x[p], y0, acc);
                } else {
                    if (!last_pass) load_y(col_cur, p + 1, y0);
                    else if (t + 1 < te) load_y(col_next, 0, y0);
                    contract(x[p], y1, acc);
                }
            }
            emit(words, acc);
            col_cur = col_next;
            col_next = col_ahead;
        };
        if constexpr (PASSES % 2 == 0) {
            for (int t = tb; t < te; ++t) tile_step(t, std::integral_constant<int, 0>{});
        } else {
            for (int t = tb; t < te; t += 2) {
                tile_step(t, std::integral_constant<int, 0>{});
                if (t + 1 < te) tile_step(t + 1, std::integral_constant<int, 1>{});
            }
        }
    } else {
        // wide rows: the features are visited in passes of 32*NV, X and Y re-read per tile and pass
        for (int t = tb; t < te; ++t) {
            if (t == wend) {
                do { ++w; wend = rwo[w + 1]; } while (wend <= t);
            }
            const int32_t row = perm_pad[(size_t)w * 16 + c];
            const int32_t col = a2b[(size_t)t * 16 + c];
            floatx4 acc{0.f, 0.f, 0.f, 0.f};
            for (int pass = 0; pass < passes; ++pass) {
                uintx4 x[NV], y[NV];
#pragma unroll
                for (int v = 0; v < NV; ++v) x[v] = uintx4{0u, 0u, 0u, 0u};
                if (row >= 0) load_row(x_base, row, pass, x);
                load_y(col, pass, y);
                contract(x, y, acc);
            }
            emit(load_words(t), acc);
        }
    }
}

// out[entry_of[q]] = packed[q] (times the value at q): packed value order -> CSR entry order
template <bool BF16>
__global__ __launch_bounds__(256) void sddmm_finish_kernel(int64_t nnz, const float* __restrict__ packed,
                                                           const int32_t* __restrict__ entry_of,
                                                           const uint16_t* __restrict__ vals, float* __restrict__ out,
                                                           int32_t use_values) {
    for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < nnz; q += (int64_t)gridDim.x * blockDim.x) {
        float v = packed[q];
        if (use_values) {
            const uint16_t a = vals[q];
            v *= BF16 ? __builtin_bit_cast(float, (uint32_t)a << 16) : (float)__builtin_bit_cast(_Float16, a);
        }
        out[entry_of[q]] = v;
    }
}

// packed[q] = csr_vals[entry_of[q]]: new values for the same pattern, CSR entry order -> packed order
__global__ __launch_bounds__(256) void repack_values_kernel(int64_t nnz, const uint16_t* __restrict__ csr_vals,
                                                            const int32_t* __restrict__ entry_of,
                                                            uint16_t* __restrict__ packed) {
    for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < nnz; q += (int64_t)gridDim.x * blockDim.x)
        packed[q] = csr_vals[entry_of[q]];
}

template <int NV, int PASSES, bool BF16>
void launch_nv(const Plan& plan, const uint16_t* X, const uint16_t* Y, const uint16_t* Y_hot, int32_t N, int32_t passes,
               float* packed_out, hipStream_t stream) {
    const DeviceFormat& f = plan.fmt;
    // without a gathered copy of Y's most used rows, a plan that kept plain entries is read through those
    const int32_t* a2b = (!Y_hot && plan.a2b_plain.p) ? plan.a2b_plain.p : f.sparse_a_to_b.p;
    const int32_t n_items = (int32_t)plan.items.size();
    const int32_t n_blocks = (n_items + kWavesPerBlock - 1) / kWavesPerBlock;
    const int blocks = ((n_blocks + 7) / 8) * 8;
    if (Y_hot)
        hipLaunchKernelGGL((sddmm_tiles_kernel<NV, PASSES, BF16, true>), dim3(blocks), dim3(kWavesPerBlock * 64), 0, stream,
                           f.row_window_offset.p, f.tc_offset.p, a2b, f.tc_local_bit.p, plan.d_perm_pad.p,
                           plan.d_items.p, X, Y, Y_hot, packed_out, n_items, n_blocks, N, passes);
    else
        hipLaunchKernelGGL((sddmm_tiles_kernel<NV, PASSES, BF16, false>), dim3(blocks), dim3(kWavesPerBlock * 64), 0,
                           stream, f.row_window_offset.p, f.tc_offset.p, a2b, f.tc_local_bit.p, plan.d_perm_pad.p,
                           plan.d_items.p, X, Y, Y_hot, packed_out, n_items, n_blocks, N, passes);
}

template <bool BF16>
void launch_typed(const Plan& plan, const uint16_t* X, const uint16_t* Y, const uint16_t* Y_hot, int32_t N, float* out,
                  int32_t use_values, hipStream_t stream) {
    float* packed = plan.sddmm_packed.p;
    switch (N) {
        case 32: launch_nv<1, 1, BF16>(plan, X, Y, Y_hot, N, 1, packed, stream); break;
        case 64: launch_nv<2, 1, BF16>(plan, X, Y, Y_hot, N, 1, packed, stream); break;
        case 96: launch_nv<3, 1, BF16>(plan, X, Y, Y_hot, N, 1, packed, stream); break;
        case 128: launch_nv<4, 1, BF16>(plan, X, Y, Y_hot, N, 1, packed, stream); break;
        case 256: launch_nv<4, 2, BF16>(plan, X, Y, Y_hot, N, 2, packed, stream); break;
        case 384: launch_nv<4, 3, BF16>(plan, X, Y, Y_hot, N, 3, packed, stream); break;
        case 512: launch_nv<4, 4, BF16>(plan, X, Y, Y_hot, N, 4, packed, stream); break;
        default: launch_nv<4, 0, BF16>(plan, X, Y, Y_hot, N, N / 128, packed, stream); break;
    }
    const int64_t nnz = plan.fmt.nnz;
    const unsigned blocks = (unsigned)std::min<int64_t>((nnz + 255) / 256, 256 * 32);
    hipLaunchKernelGGL(sddmm_finish_kernel<BF16>, dim3(blocks), dim3(256), 0, stream, nnz, packed, plan.d_entry_of.p,
                       plan.fmt.vals.p, out, use_values);
}

}  // namespace

void launch_update_values(const Plan& plan, const void* csr_vals, hipStream_t stream) {
    const int64_t nnz = plan.fmt.nnz;
    if (nnz == 0) return;
    if (!plan.d_entry_of.p) fail(ACC_SPMM_ERR_INVALID_ARG, "update_values needs a plan built with keep_entry_map = 1");
    int dev = -1;
    ACC_HIP(hipGetDevice(&dev));
    if (dev != plan.device) fail(ACC_SPMM_ERR_INVALID_ARG, "the plan lives on another device than the current one");
    const unsigned blocks = (unsigned)std::min<int64_t>((nnz + 255) / 256, 256 * 32);
    hipLaunchKernelGGL(repack_values_kernel, dim3(blocks), dim3(256), 0, stream, nnz, static_cast<const uint16_t*>(csr_vals),
                       plan.d_entry_of.p, plan.fmt.vals.p);
    ACC_HIP(hipGetLastError());
}

void launch_sddmm(const Plan& plan, const void* X, const void* Y, int32_t N, void* out, int32_t use_values,
                  hipStream_t stream) {
    const DeviceFormat& f = plan.fmt;
    if (f.WH != 16 || f.TW != 16) fail(ACC_SPMM_ERR_UNSUPPORTED, "sddmm needs a plan with 16x16 tiles");
    if (!plan.d_entry_of.p && f.nnz > 0)
        fail(ACC_SPMM_ERR_INVALID_ARG, "sddmm needs a plan built with keep_entry_map = 1");
    if (N <= 0 || N % 32 != 0 || (N > 128 && N % 128 != 0) || N > 4096)
        fail(ACC_SPMM_ERR_UNSUPPORTED, "sddmm: N must be 32, 64, 96, 128 or a multiple of 128 up to 4096");
    if ((reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(Y)) & 15)
        fail(ACC_SPMM_ERR_INVALID_ARG, "X and Y must be 16-byte aligned");
    int dev = -1;
    ACC_HIP(hipGetDevice(&dev));
    if (dev != plan.device) fail(ACC_SPMM_ERR_INVALID_ARG, "the plan lives on another device than the current one");
    if (f.nnz == 0 || plan.items.empty()) return;
    {
        std::lock_guard<std::mutex> lock(plan.workspace_mutex);
        if (!plan.sddmm_packed.p) plan.sddmm_packed.alloc((size_t)f.nnz);
    }
    // Y in the caller's order under a column order: gather its most used rows, as execute does for B
    const uint16_t* Y_hot = nullptr;
    // (as in execute, plans that also kept plain entries read all of Y in place when N <= 64)
    if (plan.d_col_order.p && plan.opt.operand_order == 0 && !(plan.a2b_plain.p && N <= 64)) {
        {
            std::lock_guard<std::mutex> lock(plan.workspace_mutex);
            if (plan.b_hot_N < N && plan.n_hot > 0) {
                plan.b_hot.alloc((size_t)plan.n_hot * (size_t)N);
                plan.b_hot_N = N;
            }
        }
        launch_permute_rows(plan.d_col_order.p, plan.n_hot, Y, plan.b_hot.p, (int64_t)N * 2, false, stream);
        Y_hot = plan.b_hot.p;
    }
    if (plan.opt.value_type == ACC_SPMM_BF16)
        launch_typed<true>(plan, static_cast<const uint16_t*>(X), static_cast<const uint16_t*>(Y), Y_hot, N,
                           static_cast<float*>(out), use_values, stream);
    else
        launch_typed<false>(plan, static_cast<const uint16_t*>(X), static_cast<const uint16_t*>(Y), Y_hot, N,
                            static_cast<float*>(out), use_values, stream);
    ACC_HIP(hipGetLastError());
}

}  // namespace accspmm
