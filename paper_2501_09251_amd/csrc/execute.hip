// Execute side of the library: picks the tile-kernel variant for a call (the kernel itself
// is in tile_kernel.hip), combines the partial tiles of split row windows (Section 3.5), and
// holds the small kernels used for comparison and calibration.
#include <algorithm>

#include <mutex>

#include "execute.h"

// Device memory for acc_spmm_execute_static: the partial tiles of split row windows and the
// gathered most used rows of B of one call.  One copy per GPU, held from the time the library
// is loaded until the process ends; host code reaches it only through the address that
// hipGetSymbolAddress returns for the current device (static_scratch_base below).
static __device__ __align__(256) unsigned char scratch[ACC_SPMM_STATIC_SCRATCH_BYTES];

namespace accspmm {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

// Sum the partial tiles of each split window and write the rows of C (Section 3.5: the
// write-back of a window shared by several work items).  One block per split window.
// narrow = 0: C is fp32.  1 / 2: C holds IEEE half / bfloat16 values (round to nearest even).
__device__ __forceinline__ uint32_t narrow_bits(float x, int narrow) {
    if (narrow == 2) {
        const uint32_t u = __builtin_bit_cast(uint32_t, x);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
        return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    }
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)x);
}

__global__ __launch_bounds__(256) void combine_split_kernel(const SplitWindow* __restrict__ splits,
                                                            const float* __restrict__ ws,
                                                            const int32_t* __restrict__ perm_pad,
                                                            void* __restrict__ C_any, int32_t N, int32_t narrow) {
    const SplitWindow sw = splits[blockIdx.x];
    float* const C = static_cast<float*>(C_any);
    uint16_t* const C16 = static_cast<uint16_t*>(C_any);
    if (N & 3) {  // rows of C are not 16-byte aligned: one value at a time
        for (int e = threadIdx.x; e < 16 * N; e += blockDim.x) {
            const int r = e / N, j = e - r * N;
            const int row = perm_pad[(size_t)sw.window * 16 + r];
            if (row < 0) continue;
            float s = 0.f;
            for (int slot = sw.slot_begin; slot < sw.slot_end; ++slot) s += ws[((size_t)slot * 16 + r) * (size_t)N + j];
            if (narrow) C16[(size_t)row * (size_t)N + j] = (uint16_t)narrow_bits(s, narrow);
            else __builtin_nontemporal_store(s, C + (size_t)row * (size_t)N + j);
        }
        return;
    }
    const int n4 = N >> 2;
    for (int e = threadIdx.x; e < 16 * n4; e += blockDim.x) {
        const int r = e / n4, j = (e - r * n4) << 2;
        const int row = perm_pad[(size_t)sw.window * 16 + r];
        if (row < 0) continue;
        floatx4 s{0.f, 0.f, 0.f, 0.f};
        for (int slot = sw.slot_begin; slot < sw.slot_end; ++slot)
            s += *reinterpret_cast<const floatx4*>(ws + ((size_t)slot * 16 + r) * (size_t)N + j);
        if (narrow) {
            typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));
            const uintx2 v{narrow_bits(s[0], narrow) | (narrow_bits(s[1], narrow) << 16),
                           narrow_bits(s[2], narrow) | (narrow_bits(s[3], narrow) << 16)};
            *reinterpret_cast<uintx2*>(C16 + (size_t)row * (size_t)N + j) = v;
        } else {
            __builtin_nontemporal_store(s, reinterpret_cast<floatx4*>(C + (size_t)row * (size_t)N + j));
        }
    }
}

// Baseline: one wavefront per CSR row, lanes over the N features, serial loop over the
// row's entries, fp32 FMA.
__global__ __launch_bounds__(256) void csr_row_per_wave_kernel(int64_t M, const int32_t* __restrict__ rowptr,
                                                               const int32_t* __restrict__ colidx,
                                                               const uint16_t* __restrict__ vals,
                                                               const uint16_t* __restrict__ B,
                                                               float* __restrict__ C, int32_t N, int32_t bf16) {
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    auto widen = [bf16](uint16_t h) -> float {
        return bf16 ? __builtin_bit_cast(float, (uint32_t)h << 16) : (float)__builtin_bit_cast(_Float16, h);
    };
    if (row >= M) return;
    const int lane = threadIdx.x & 63;
    const int pb = rowptr[row], pe = rowptr[row + 1];
    for (int j0 = 0; j0 < N; j0 += 64) {
        const int j = j0 + lane;
        float acc = 0.f;
        if (j < N)
            for (int q = pb; q < pe; ++q) {
                const float a = widen(vals[q]);
                const float b = widen(B[(size_t)colidx[q] * (size_t)N + j]);
                acc = __builtin_fmaf(a, b, acc);
            }
        if (j < N) C[(size_t)row * (size_t)N + j] = acc;
    }
}

__global__ __launch_bounds__(256) void calibration_copy_kernel(uintx4* __restrict__ dst, const uintx4* __restrict__ src,
                                                               size_t n16) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

// Address of `scratch` on device `dev`, which must be the current device.  Every GPU has its own
// copy of the array at its own address; it is looked up once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_base[kMaxDevices] = {};

unsigned char* static_scratch_base(int dev) {
    if (dev < 0 || dev >= kMaxDevices) fail(ACC_SPMM_ERR_UNSUPPORTED, "device index beyond the static scratch table");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_base[dev]) {
        void* ptr = nullptr;
        ACC_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) fail(ACC_SPMM_ERR_HIP, "hipGetSymbolAddress returned no address for the static scratch array");
        g_scratch_base[dev] = static_cast<unsigned char*>(ptr);
    }
    return g_scratch_base[dev];
}

// A call that would have to allocate while its stream is being captured into a graph fails
// instead: hipMalloc / hipFree are not legal there, and hipFree would wait for the device.
void refuse_allocation_under_capture(hipStream_t stream, const char* what) {
    if (!stream) return;
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &status) != hipSuccess || status != hipStreamCaptureStatusNone)
        fail(ACC_SPMM_ERR_INVALID_ARG,
             std::string("the stream is being captured and this call would have to allocate ") + what +
                 ": run one call at this N outside the capture first, or use acc_spmm_execute_static");
}

// Measurement aid: nothing but the memory pattern of the tile kernel's B gather.  A wavefront walks
// its share of `index` sixteen entries (one "tile") at a time; each 16-lane group reads four of the
// sixteen rows, 16 bytes per lane, so that sixteen lanes cover 256 contiguous bytes of a row (wider
// rows in further steps of 256 bytes).  Four tiles are requested before the first is consumed.  With
// write_rows > 0 the wave also writes write_rows rows of row_u4 * 32 bytes (the fp32 image of a
// row) after every write_every tiles, as the tile kernel writes a window of C after its tiles.
__global__ __launch_bounds__(256) void calibration_gather_kernel(const uintx4* __restrict__ table, int64_t row_u4,
                                                                 const int32_t* __restrict__ index, int64_t n_tiles,
                                                                 uintx4* __restrict__ sink, uintx4* __restrict__ out,
                                                                 int32_t write_every, int32_t write_rows) {
    const int lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), n_waves = (int64_t)gridDim.x * 4;
    const int64_t per_wave = (n_tiles + n_waves - 1) / n_waves;
    const int64_t t_begin = wave * per_wave, t_end = t_begin + per_wave < n_tiles ? t_begin + per_wave : n_tiles;
    typedef int32_t intx4 __attribute__((ext_vector_type(4)));
    uintx4 acc{0u, 0u, 0u, 0u};
    int64_t written = 0;
    for (int64_t t = t_begin; t < t_end; t += 4) {
        intx4 ids[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int64_t tt = t + k < t_end ? t + k : t_end - 1;
            ids[k] = *reinterpret_cast<const intx4*>(index + tt * 16 + 4 * g);
        }
        for (int64_t u = c; u < row_u4; u += 16) {
            uintx4 v[16];
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int q = 0; q < 4; ++q) v[4 * k + q] = table[(int64_t)ids[k][q] * row_u4 + u];
#pragma unroll
            for (int k = 0; k < 16; ++k) acc ^= v[k];
        }
        if (write_rows > 0 && (t - t_begin) % write_every == 0) {   // write_every is a multiple of 4
            // rows of the output stream owned by this wave, consecutive, each row_u4 * 2 units of 16 bytes
            const int64_t units = (int64_t)write_rows * row_u4 * 2;
            uintx4* dst = out + (wave * ((per_wave + write_every - 1) / write_every) * (int64_t)write_rows * row_u4 * 2) + written;
            for (int64_t e = lane; e < units; e += 64) dst[e] = acc;
            written += units;
        }
    }
    sink[(int64_t)blockIdx.x * 256 + threadIdx.x] = acc;   // keeps the loads alive; 16 bytes per lane
}

}  // namespace

void launch_calibration_gather(const void* table, int64_t rows, int64_t row_bytes, const int32_t* index, int64_t n_index,
                               void* sink, size_t sink_bytes, void* out, size_t out_bytes, int32_t write_every,
                               int32_t write_rows, hipStream_t stream) {
    if (!table || !index || !sink || rows <= 0 || row_bytes <= 0 || (row_bytes & 15) || n_index <= 0 || (n_index & 15) ||
        ((reinterpret_cast<uintptr_t>(table) | reinterpret_cast<uintptr_t>(index) | reinterpret_cast<uintptr_t>(sink) |
          reinterpret_cast<uintptr_t>(out)) & 15))
        fail(ACC_SPMM_ERR_INVALID_ARG, "calibration gather needs 16-byte aligned pointers, rows of a multiple of 16 bytes "
                                       "and a multiple of 16 index entries");
    const int64_t n_tiles = n_index / 16;
    const unsigned blocks = (unsigned)std::min<int64_t>((n_tiles + 3) / 4, 256 * 16);
    if (sink_bytes < (size_t)blocks * 256 * 16) fail(ACC_SPMM_ERR_INVALID_ARG, "calibration gather: sink smaller than 16 MiB");
    if (write_rows > 0) {
        if (!out || write_every <= 0 || (write_every & 3))
            fail(ACC_SPMM_ERR_INVALID_ARG, "calibration gather: with write_rows, out must be given and write_every a positive multiple of 4");
        const int64_t n_waves = (int64_t)blocks * 4, per_wave = (n_tiles + n_waves - 1) / n_waves;
        const int64_t bursts = (per_wave + write_every - 1) / write_every;
        const size_t need = (size_t)n_waves * (size_t)bursts * (size_t)write_rows * (size_t)row_bytes * 2;
        if (out_bytes < need)
            fail(ACC_SPMM_ERR_INVALID_ARG, "calibration gather: out must hold " + std::to_string(need) + " bytes");
    }
    hipLaunchKernelGGL(calibration_gather_kernel, dim3(blocks), dim3(256), 0, stream, static_cast<const uintx4*>(table),
                       row_bytes / 16, index, n_tiles, static_cast<uintx4*>(sink), static_cast<uintx4*>(out), write_every,
                       write_rows);
    ACC_HIP(hipGetLastError());
}

void prepare_static_scratch() {
    int dev = -1;
    ACC_HIP(hipGetDevice(&dev));
    (void)static_scratch_base(dev);
}

void launch_execute(const Plan& plan, const void* B, int32_t N, void* C, hipStream_t stream, float* tiles_ms,
                    float* combine_ms, float* gather_ms, bool narrow_c, bool static_scratch) {
    const bool timed = tiles_ms != nullptr;
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
    if (timed) {
        *tiles_ms = 0.f;
        if (combine_ms) *combine_ms = 0.f;
        if (gather_ms) *gather_ms = 0.f;
        for (auto& e : ev) ACC_HIP(hipEventCreate(&e));
    }
    struct EventGuard {
        hipEvent_t* ev;
        ~EventGuard() { for (int i = 0; i < 4; ++i) if (ev[i]) (void)hipEventDestroy(ev[i]); }
    } guard{ev};
    const DeviceFormat& f = plan.fmt;
    if (f.WH != 16 || (f.TW != 16 && f.TW != 32))
        fail(ACC_SPMM_ERR_UNSUPPORTED, "execute needs a plan with 16x16 or 16x32 tiles");
    const bool tw32 = f.TW == 32;
    if (tw32 && (int64_t)f.vals.n < f.nnz + 10)
        fail(ACC_SPMM_ERR_UNSUPPORTED, "this plan's value array lacks the slack that the 16x32 kernel's loads need");
    if (N <= 0 || N > kMaxN) fail(ACC_SPMM_ERR_UNSUPPORTED, "N must be between 1 and 65536");
    if ((reinterpret_cast<uintptr_t>(B) | reinterpret_cast<uintptr_t>(C)) & 15)
        fail(ACC_SPMM_ERR_INVALID_ARG, "B and C must be 16-byte aligned");
    if (f.M == 0) return;
    int dev = -1;
    ACC_HIP(hipGetDevice(&dev));
    if (dev != plan.device) fail(ACC_SPMM_ERR_INVALID_ARG, "the plan lives on another device than the current one");
    // Column order with B in the caller's order: gather the most used rows and read the rest in place,
    // unless the plan also kept plain entries and this call's rows are narrow (the gathered copy needs
    // 64-bit addressing, which costs more than it gains at N <= 64 on plans of that size).
    const bool hot_entries = plan.d_col_order.p != nullptr && plan.opt.operand_order == 0 && f.nnz > 0;
    const bool gather = hot_entries && !(plan.a2b_plain.p != nullptr && N <= 64);
    float* ws = nullptr;          // partial tiles of split windows, n_slots x 16 x N
    uint16_t* b_hot = nullptr;    // gathered most used rows of B, n_hot x N
    const size_t ws_bytes = (size_t)plan.n_slots * 16 * (size_t)N * sizeof(float);
    const size_t hot_bytes = (gather && plan.n_hot > 0) ? (size_t)plan.n_hot * (size_t)N * sizeof(uint16_t) : 0;
    if (static_scratch) {
        // both buffers inside the library's static device array; nothing is allocated
        const size_t ws_span = (ws_bytes + 255) & ~(size_t)255;
        if (ws_span + hot_bytes > (size_t)ACC_SPMM_STATIC_SCRATCH_BYTES)
            fail(ACC_SPMM_ERR_UNSUPPORTED,
                 "acc_spmm_execute_static: this plan at this N needs " + std::to_string(ws_span + hot_bytes) +
                     " bytes of scratch memory (split-window partial tiles + gathered rows of B), the static buffer holds " +
                     std::to_string((size_t)ACC_SPMM_STATIC_SCRATCH_BYTES) + "; use acc_spmm_execute");
        unsigned char* base = static_scratch_base(dev);
        ws = reinterpret_cast<float*>(base);
        b_hot = reinterpret_cast<uint16_t*>(base + ws_span);
    } else {
        // grown only when a wider N arrives; hipFree inside alloc() waits for kernels still using the old buffer
        std::lock_guard<std::mutex> lock(plan.workspace_mutex);
        if (plan.n_slots > 0 && plan.workspace_N < N) {
            refuse_allocation_under_capture(stream, "the partial-tile workspace of the split row windows");
            plan.workspace.alloc((size_t)plan.n_slots * 16 * (size_t)N);
            plan.workspace_N = N;
        }
        if (hot_bytes > 0 && plan.b_hot_N < N) {
            refuse_allocation_under_capture(stream, "the buffer for the gathered rows of B");
            plan.b_hot.alloc((size_t)plan.n_hot * (size_t)N);
            plan.b_hot_N = N;
        }
        ws = plan.workspace.p;
        b_hot = plan.b_hot.p;
    }
    if (timed) ACC_HIP(hipEventRecord(ev[3], stream));
    if (gather) launch_permute_rows(plan.d_col_order.p, plan.n_hot, B, b_hot, (int64_t)N * 2, false, stream);
    ExecParams p;
    p.rwo = f.row_window_offset.p;
    p.tco = f.tc_offset.p;
    p.a2b = (hot_entries && !gather) ? plan.a2b_plain.p : f.sparse_a_to_b.p;
    p.bits = f.tc_local_bit.p;
    p.vals = f.vals.p;
    p.perm_pad = plan.d_perm_pad.p;
    p.items = plan.d_items.p;
    p.B = static_cast<const uint16_t*>(B);
    p.C = static_cast<float*>(C);
    p.ws = ws;
    p.n_items = (int32_t)plan.items.size();
    p.n_blocks = (p.n_items + kWavesPerBlock - 1) / kWavesPerBlock;
    p.N = N;
    p.B_hot = b_hot;
    p.addr = gather ? kAddrHot
                    : ((plan.stats.K >= (1 << 24) || (int64_t)plan.stats.K * N * 2 >= ((int64_t)1 << 32)) ? kAddrWide
                                                                                                        : kAddrNarrow);
    // Shape of the launch: FPL features per lane (a divisor of N, so that vector loads stay
    // aligned and no lane straddles N, and no wider than N needs), 16*FPL features per slab,
    // one or two slabs per wave, the rest of N over gridDim.y.
    const int fpl_fit = N > 64 ? 8 : (N > 32 ? 4 : (N > 16 ? 2 : 1));
    const int fpl_div = (N % 8 == 0) ? 8 : ((N % 4 == 0) ? 4 : ((N % 2 == 0) ? 2 : 1));
    p.fpl = std::min(fpl_fit, fpl_div);
    const int slab_width = 16 * p.fpl;
    const int slabs = (N + slab_width - 1) / slab_width;
    // Two slabs per wave halve the reads of A and of the index words; one slab per wave with twice the waves
    // keeps more rows of B in flight and needs fewer registers.  Measured at N = 256 and 512: one slab is 6-15 %
    // faster on sparse tiles with the two-matrix addressing of a column order (balanced power-law inputs; that
    // addressing costs registers), two slabs are 3-11 % faster on sparse tiles read in place and 8-15 % on dense tiles.
    const bool dense_tiles = plan.stats.mean_nnz_per_tile * 16.0 / f.TW >= 24.0;   // per 16 x 16 positions
    p.ns = ((dense_tiles || p.addr != kAddrHot) && (slabs % 2 == 0 || slabs > 3)) ? 2 : 1;
    if (plan.opt.slabs_per_wave == 1) p.ns = 1;
    if (plan.opt.slabs_per_wave == 2 && slabs >= 2) p.ns = 2;
    p.grid_y = (slabs + p.ns - 1) / p.ns;
    p.tail = (int64_t)p.grid_y * p.ns * slab_width != N;
    if (!p.tail && p.ns == 2 && p.fpl != 8) p.tail = true;  // shape compiled only in its general form
    // How the packed values reach the lanes (see the tile kernel's header), by what measured fastest on
    // uniform, power-law, stencil and block inputs at N = 16 .. 512: lanes of one or two features (N <= 32)
    // read their span; lanes of four features (N <= 64) share one cooperative read when tiles are
    // dense (24 entries per tile on average: the break-even lay between 18 and 35) or the launch has enough tiles to
    // be bound by throughput rather than by the latency of one wave's chain of tiles; 16-byte lanes read
    // their span when tiles are dense or a wave's chain of tiles is short (fewer than 64 tiles per work item: inputs
    // that need no load balancing, one window per wave), and value by value on the long chains of sparse tiles that
    // balanced power-law inputs give (there the span read measured 1-4 % slower, on the short chains 11 % faster).
    const bool many_tiles = plan.stats.num_tiles >= 16384;
    // tiles a wave multiplies one after the other: a window or two without load balancing, hundreds with it
    const bool short_chains = plan.stats.num_tiles < 64 * (int64_t)plan.items.size();
    // gathered rows of B per entry of A: near 1 when the rows of a window share almost no columns.  At N <= 32 the
    // span read's lead over the per-lane loads shrinks as this grows (twelve inputs: 22 % at 0.87, 7-15 % at 0.91,
    // 2 % at 0.97) and is a loss of 4-10 % at 0.96 on long chains of tiles
    const bool unshared_rows = (double)plan.stats.sum_distinct_cols >= 0.95 * (double)std::max<int64_t>(1, f.nnz);
    switch (plan.opt.value_fetch) {
        case 1: p.fetch = kFetchLane; break;
        case 2: p.fetch = kFetchCoop; break;
        case 3: p.fetch = kFetchSpan; break;
        default:
            if (p.fpl <= 2) p.fetch = (!short_chains && unshared_rows) ? kFetchLane : kFetchSpan;
            else if (p.fpl == 4) p.fetch = (dense_tiles || many_tiles) ? kFetchCoop : kFetchLane;
            else p.fetch = (dense_tiles || short_chains) ? kFetchSpan : kFetchLane;
    }
    if (p.fetch == kFetchSpan && (int64_t)f.vals.n < f.nnz + 6) p.fetch = kFetchLane;   // a plan file without the slack
    p.tw32 = tw32;
    if (tw32) p.fetch = kFetchSpan;   // the only way the 16 x 32 kernel fetches values
    // Tiles in flight per wave: swept on long chains of tiles (balanced power-law inputs), where 3 is best for one
    // 128-feature slab and 2 otherwise (narrower lanes: 2-5 % faster than 1 on three of four such inputs at
    // N = 32 and 64, 2 % slower on the fourth); a wave that multiplies one window's dozen tiles and ends
    // gains nothing from a deep ring and pays its prologue (held-out inputs: 4-10 % faster at depth 1).
    const int default_depth = short_chains ? 1 : ((p.fpl == 8 && p.ns == 1) ? 3 : 2);
    p.depth = plan.opt.no_prefetch ? 0 : (plan.opt.pipeline_depth > 0 ? plan.opt.pipeline_depth : default_depth);
    if (tw32) {
        // a tile holds twice the rows of B: half the depth keeps the same bytes in flight; depths 1 and 2 exist
        if (plan.opt.no_prefetch) fail(ACC_SPMM_ERR_UNSUPPORTED, "plans with 16x32 tiles run with prefetch only");
        p.depth = plan.opt.pipeline_depth > 0 ? std::min(plan.opt.pipeline_depth, 2) : (default_depth >= 3 ? 2 : 1);
    }
    p.store_mode = (plan.opt.streaming_stores != 0 ? kStoreStreaming : 0) | (narrow_c ? kStoreNarrow : 0);
    p.bf16 = plan.opt.value_type == ACC_SPMM_BF16;
    p.lds = plan.opt.lds_staging != 0;
    if (p.lds) {
        // the comparison form exists for whole slabs of at least two features per lane, one slab per wave
        if (p.fpl < 2 || p.ns != 1 || p.tail || p.bf16 || plan.opt.no_prefetch || tw32)
            fail(ACC_SPMM_ERR_UNSUPPORTED, "lds_staging runs fp16 plans at N = 32, 64 or an odd multiple of 128 up to 384, with prefetch");
        p.depth = 1;   // a double buffer: one tile ahead
    }
    if (timed) ACC_HIP(hipEventRecord(ev[0], stream));
    if (p.n_items > 0) {
        switch (p.fpl * 2 + (p.bf16 ? 1 : 0)) {
            case 2: launch_tiles_f1_t0(p, stream); break;
            case 3: launch_tiles_f1_t1(p, stream); break;
            case 4: launch_tiles_f2_t0(p, stream); break;
            case 5: launch_tiles_f2_t1(p, stream); break;
            case 8: launch_tiles_f4_t0(p, stream); break;
            case 9: launch_tiles_f4_t1(p, stream); break;
            case 16: launch_tiles_f8_t0(p, stream); break;
            default: launch_tiles_f8_t1(p, stream); break;
        }
        ACC_HIP(hipGetLastError());
    }
    if (timed) ACC_HIP(hipEventRecord(ev[1], stream));
    if (!plan.splits.empty()) {
        hipLaunchKernelGGL(combine_split_kernel, dim3((unsigned)plan.splits.size()), dim3(256), 0, stream,
                           plan.d_splits.p, ws, plan.d_perm_pad.p, C, N,
                           narrow_c ? (plan.opt.value_type == ACC_SPMM_BF16 ? 2 : 1) : 0);
        ACC_HIP(hipGetLastError());
    }
    if (timed) {
        ACC_HIP(hipEventRecord(ev[2], stream));
        ACC_HIP(hipEventSynchronize(ev[2]));
        ACC_HIP(hipEventElapsedTime(tiles_ms, ev[0], ev[1]));
        if (combine_ms && !plan.splits.empty()) ACC_HIP(hipEventElapsedTime(combine_ms, ev[1], ev[2]));
        if (gather_ms && gather) ACC_HIP(hipEventElapsedTime(gather_ms, ev[3], ev[0]));
    }
}

void launch_calibration_copy(void* dst, const void* src, size_t bytes, hipStream_t stream) {
    if (!dst || !src || (bytes & 15) || ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15))
        fail(ACC_SPMM_ERR_INVALID_ARG, "calibration copy needs 16-byte aligned pointers and size");
    if (!bytes) return;
    const size_t n16 = bytes / 16;
    const unsigned blocks = (unsigned)std::min<size_t>((n16 + 255) / 256, 256 * 64);
    hipLaunchKernelGGL(calibration_copy_kernel, dim3(blocks), dim3(256), 0, stream, static_cast<uintx4*>(dst),
                       static_cast<const uintx4*>(src), n16);
    ACC_HIP(hipGetLastError());
}

void launch_csr_naive(const Plan& plan, const void* B, int32_t N, void* C, hipStream_t stream) {
    if (!plan.d_rowptr.p) fail(ACC_SPMM_ERR_INVALID_ARG, "plan was built without keep_csr");
    if (N <= 0) fail(ACC_SPMM_ERR_INVALID_ARG, "N must be positive");
    const int64_t M = plan.fmt.M;
    if (M == 0) return;
    hipLaunchKernelGGL(csr_row_per_wave_kernel, dim3((unsigned)((M + 3) / 4)), dim3(256), 0, stream, M,
                       plan.d_rowptr.p, plan.d_colidx.p, plan.d_vals.p, static_cast<const uint16_t*>(B),
                       static_cast<float*>(C), N, (int32_t)(plan.opt.value_type == ACC_SPMM_BF16));
    ACC_HIP(hipGetLastError());
}

}  // namespace accspmm
