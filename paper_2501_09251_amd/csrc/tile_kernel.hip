// Runtime kernels: C = A.B from the bitmap tile format (paper Section 3.4, Algorithm 2,
// re-designed for gfx950).
//
// One wavefront owns one work item: a run of whole row windows, or a slice of the tiles of
// one heavy window (Section 3.5).  For every 16x16 tile the wavefront
//   - reads the tile's 16 SparseAToB entries and gathers those 16 rows of B straight into
//     registers (as in the paper's Section 3.4, B goes global -> registers): each 16-lane group
//     reads four whole rows with 16-byte loads per lane,
//   - decodes its own four positions of the tile from the bitmap (popcount of the lower
//     bits gives the value offset, Section 3.3) and reads up to four packed values,
//   - issues v_mfma_f32_16x16x16_f16 with the sparse tile as the 16x16 left operand and
//     sixteen feature columns of the gathered rows as the right operand.
// Lane c of a group owns features [FPL*c, FPL*c+FPL) of a 16*FPL-wide slab, so a feature's
// position inside an MFMA is a free choice and no transpose through LDS is needed: the
// four k-values of one feature come from four registers and are packed with v_perm_b32.
//
// The packed values of a tile reach the lanes in one of three ways (template FETCH).  Per-lane
// (kFetchLane): each lane reads its up-to-four values itself (four 2-byte loads).  Cooperative
// (kFetchCoop): the wave reads the tile's contiguous values once, one dword per lane, and every
// lane then picks its values out of the other lanes' registers with ds_bpermute.  Span
// (kFetchSpan): a lane's values are consecutive in the packed array (row-major inside the tile),
// so the lane reads the three dwords that hold its first value and the three after it with one
// load, shifts by the odd half and routes the halves to its set bits with the byte permutes of
// the cooperative way; the array is allocated with eight values of slack so that the load never
// leaves it.  (The same eight bytes as one load aligned to two bytes only measured slower.)
// Execute selects the way from the lane width, the plan's mean entries per tile and N.
//
// Loads are software-pipelined (the "least bubble" idea of Section 3.4): the B rows and
// values of tiles t+1..t+DEPTH are in flight while tile t is multiplied, and the index
// words of tile t+DEPTH+1 are requested one step before they are needed for addresses.
//
// LDS = true is the staging that the paper's Algorithm 2 describes, for comparison: the B rows of the
// next tile go from global memory straight into LDS (global_load_lds, no registers in between) while
// the current tile, read back from the other LDS buffer, is multiplied: a double buffer, one tile
// ahead.  The register ring above measured as fast or faster on every workload and stays the default.
//
// TW32 = true runs plans whose tiles are 16 x 32 (tile_width = 32) on v_mfma_f32_16x16x32_f16: a lane
// group gathers eight rows of B per tile, a lane's sparse operand is the eight positions (row c,
// k = 8g .. 8g+7), i.e. one byte of the row's 32-bit bitmap word, which the lane loads itself (a
// row is exactly one dword; the offset of the row's first value is a prefix sum of popcounts over
// the sixteen lanes of a group, by DPP row shifts), and the values come by two span loads, one per
// nibble.  Half as many tiles, index-word requests and window tests for the same columns; the
// padding of a window's last tile grows.
//
// This file is compiled once per (features per lane, value type): ACC_TILE_FPL in {1, 2, 4, 8}
// and ACC_TILE_BF16 in {0, 1} come from the command line, so that the many instantiations
// build in parallel.
#include <type_traits>

#include "execute.h"

#if !defined(ACC_TILE_FPL) || !defined(ACC_TILE_BF16)
#error "compile with -DACC_TILE_FPL=<1|2|4|8> -DACC_TILE_BF16=<0|1>"
#endif

namespace accspmm {
namespace {

typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));
typedef int32_t intx4 __attribute__((ext_vector_type(4)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bfloat8 __attribute__((ext_vector_type(8)));

template <int FPL>
struct Chunk {  // FPL consecutive fp16 features of one B row, as dwords
    static constexpr int DW = (FPL + 1) / 2;
    uint32_t d[DW];
};

template <int FPL>
__device__ __forceinline__ void load_chunk(const uint16_t* p, Chunk<FPL>& c) {
    if constexpr (FPL == 8) {
        uintx4 v = *reinterpret_cast<const uintx4*>(p);
        c.d[0] = v.x; c.d[1] = v.y; c.d[2] = v.z; c.d[3] = v.w;
    } else if constexpr (FPL == 4) {
        uintx2 v = *reinterpret_cast<const uintx2*>(p);
        c.d[0] = v.x; c.d[1] = v.y;
    } else if constexpr (FPL == 2) {
        c.d[0] = *reinterpret_cast<const uint32_t*>(p);
    } else {
        c.d[0] = *p;
    }
}

// The same from a 64-bit byte address known to be in global memory.  A pointer made from an
// integer is a generic one to the compiler, and generic (flat) loads count on both the vector
// and the scalar/LDS wait counters, so that every wait for a scalar load would also drain the
// B rows in flight; naming the address space keeps them on the vector counter alone.
template <int FPL>
__device__ __forceinline__ void load_chunk_global(uint64_t addr, Chunk<FPL>& c) {
#define ACC_GLOBAL(T) reinterpret_cast<const __attribute__((address_space(1))) T*>(addr)
    if constexpr (FPL == 8) {
        uintx4 v = *ACC_GLOBAL(uintx4);
        c.d[0] = v.x; c.d[1] = v.y; c.d[2] = v.z; c.d[3] = v.w;
    } else if constexpr (FPL == 4) {
        uintx2 v = *ACC_GLOBAL(uintx2);
        c.d[0] = v.x; c.d[1] = v.y;
    } else if constexpr (FPL == 2) {
        c.d[0] = *ACC_GLOBAL(uint32_t);
    } else {
        c.d[0] = *ACC_GLOBAL(uint16_t);
    }
#undef ACC_GLOBAL
}

// fp32 -> the 16-bit type of the plan (IEEE half or bfloat16), round to nearest even, as bits
template <bool BF16>
__device__ __forceinline__ uint32_t narrow16(float x) {
    if constexpr (BF16) {
        const uint32_t u = __builtin_bit_cast(uint32_t, x);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;  // nan stays nan
        return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    } else {
        return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)x);
    }
}

template <bool TW32>
struct TileMeta {       // index words of one 16 x 16 tile
    intx4 cols;         // this lane group's four SparseAToB entries
    uint64_t bm[4];     // TCLocalBit (wave-uniform)
    int32_t tco;        // TCOffset (wave-uniform)
};
template <>
struct TileMeta<true> { // index words of one 16 x 32 tile
    intx4 cols, cols2;  // this lane group's eight SparseAToB entries
    uint32_t rowbits;   // TCLocalBit: the 32 bits of this lane's row c
    int32_t tco;        // TCOffset (wave-uniform)
};

template <int FPL, int NS, int QR>
struct TileData {       // what the multiply needs; QR = rows of B per lane group and tile
    Chunk<FPL> b[NS][QR];
    // per-lane fetch: v[0..3] = up to four packed values (fp16 bits).
    // cooperative fetch: v[0..2] = the tile's packed values, chunk k's dword L in lane L;
    //                    v[3] = index of this lane's first value relative to the first loaded half
    // span fetch: v[0..2] = the dwords around this lane's four values, v[3] = 0 or 16, the bit where they start
    //             (16 x 32 tiles: v[4..7] = the same for the values of the upper nibble)
    uint32_t v[QR];
    uint32_t nib;       // this lane's four (eight) bitmap bits
    uint32_t nchunk;    // cooperative fetch: 64-dword chunks that hold values (wave-uniform)
};

// The index arrays are passed as separate const __restrict__ kernel arguments (not inside a
// struct) so that the compiler knows they are read-only and wave-uniform accesses to them
// become scalar loads.
// ADDR = kAddrNarrow: B is smaller than 4 GiB and K < 2^24, so a B row's byte offset is formed
// with one 24-bit multiply in 32 bits and added to the uniform base by the load itself.
// kAddrWide: 64-bit row offsets.  kAddrHot: a SparseAToB entry h < 0 names row ~h of a second,
// small matrix (the plan's copy of the most used rows of B, gathered together); entries >= 0 are
// rows of B as before; 64-bit addresses.
// TAIL = true: N is not a whole number of this kernel's feature slabs (16*FPL features per slab,
// NS slabs per wave, gridDim.y waves per item); lanes whose features lie at or beyond N neither
// load nor store.  N is always a multiple of FPL, so a lane is wholly inside or wholly outside.
// BF16 = true: the 16-bit values of A and B are bfloat16 instead of IEEE half; only the MFMA
// instruction differs, the data movement is the same.
template <int FPL, int NS, int DEPTH, int ADDR, int FETCH, bool TAIL, bool BF16, bool LDS = false, bool TW32 = false>
__global__ __launch_bounds__(kWavesPerBlock * 64) void spmm_tiles_kernel(
    const int32_t* __restrict__ g_rwo, const int32_t* __restrict__ g_tco, const int32_t* __restrict__ g_a2b,
    const uint64_t* __restrict__ g_bits, const uint16_t* __restrict__ g_vals, const int32_t* __restrict__ g_perm_pad,
    const WorkItem* __restrict__ g_items, const uint16_t* __restrict__ g_B, const uint16_t* __restrict__ g_Bhot,
    float* __restrict__ g_C, float* __restrict__ g_ws, int32_t n_items, int32_t n_blocks, int32_t N_arg,
    int32_t store_mode) {
    constexpr int R = DEPTH + 1;
    constexpr int SW = 16 * FPL;  // features per slab
    static_assert(!LDS || (DEPTH == 1 && NS == 1 && !TAIL && FPL >= 2 && !TW32), "LDS staging: double buffer, whole slabs, dword lanes");
    static_assert(!TW32 || FETCH == kFetchSpan, "16 x 32 tiles fetch their values by span");
    constexpr int QR = TW32 ? 8 : 4;     // rows of B per lane group and tile
    // LDS staging: per wave and ring slot, four planes (one per B row of the lane group) of 64 lanes x
    // DW dwords, each dword column a plane of its own when a lane holds fewer than four (the load
    // instruction places lane l's data at l times its size)
    constexpr int DW = Chunk<FPL>::DW;
    __shared__ uint32_t stage[LDS ? kWavesPerBlock * R * 4 * DW * 64 : 1];
    uint32_t* const stage_wave = stage + (LDS ? (threadIdx.x >> 6) * (R * 4 * DW * 64) : 0);
    struct {
        const int32_t* __restrict__ rwo; const int32_t* __restrict__ tco; const int32_t* __restrict__ a2b;
        const uint64_t* __restrict__ bits; const uint16_t* __restrict__ vals; const int32_t* __restrict__ perm_pad;
        const WorkItem* __restrict__ items; const uint16_t* __restrict__ B; float* __restrict__ C; float* __restrict__ ws;
        int32_t n_items, n_blocks, N;
    } p{g_rwo, g_tco, g_a2b, g_bits, g_vals, g_perm_pad, g_items, g_B, g_C, g_ws, n_items, n_blocks, N_arg};
    const int lane = threadIdx.x & 63;
    const int g = lane >> 4, c = lane & 15;
    // Consecutive blocks go to different XCDs (round-robin over 8); give each XCD one
    // contiguous eighth of the items so that neighbouring windows share an L2.
    const int per_xcd = (p.n_blocks + 7) >> 3;
    const int lblock = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (lblock >= p.n_blocks) return;
    const int item_id = __builtin_amdgcn_readfirstlane(lblock * kWavesPerBlock + (int)(threadIdx.x >> 6));
    if (item_id >= p.n_items) return;
    const WorkItem it = p.items[item_id];
    const int w_begin = __builtin_amdgcn_readfirstlane(it.w_begin);
    const int w_end_raw = __builtin_amdgcn_readfirstlane(it.w_end);
    const int tb = __builtin_amdgcn_readfirstlane(it.t_begin);
    const int te = __builtin_amdgcn_readfirstlane(it.t_end);
    const bool partial = w_end_raw < 0;
    const int w_end = partial ? w_begin + 1 : w_end_raw;
    const int N = p.N;
    const int f0 = (int)(blockIdx.y * NS) * SW + c * FPL;  // this lane's first feature in slab 0 of this wave
    bool act[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) act[s] = !TAIL || (f0 + s * SW < N);
    const bool nt = (store_mode & kStoreStreaming) != 0;
    const bool c16 = (store_mode & kStoreNarrow) != 0;  // C holds 16-bit values of the plan's type

    // lane constants of the bitmap decode: bit index of (row c, k 4g) is c*16 + 4g
    const int wq = c >> 2;
    const int sh = ((c & 3) << 4) | (g << 2);
    const uint64_t below_mask = (1ull << sh) - 1ull;
    const bool w1 = wq >= 1, w2 = wq >= 2, w3 = wq >= 3;
    // Cooperative fetch: byte-permute selectors, entry (lane & 15) = a pattern of four bits.  Output
    // half j is half popcount(bits below j) of the lane's four consecutive values if bit j is set
    // (bytes 2k, 2k+1), else the constant zero (selector byte 0x0c).
    constexpr bool COOP = FETCH == kFetchCoop;
    constexpr bool SPAN = FETCH == kFetchSpan;
    uint32_t lut_lo = 0, lut_hi = 0;
    if constexpr (COOP || SPAN) {
        const uint32_t pat = (uint32_t)lane & 15u;
        uint32_t sel[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t k = (uint32_t)__builtin_popcount(pat & ((1u << j) - 1u));
            sel[j] = ((pat >> j) & 1u) ? (((2u * k + 1u) << 8) | (2u * k)) : 0x0c0cu;
        }
        lut_lo = sel[0] | (sel[1] << 16);
        lut_hi = sel[2] | (sel[3] << 16);
    }

    floatx4 acc[NS][FPL];
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int m = 0; m < FPL; ++m) acc[s][m] = floatx4{0.f, 0.f, 0.f, 0.f};

    // Rows of C owned by this lane for the window being accumulated (requested when the window
    // starts, so that closing the window does not wait on a fresh load).
    intx4 rows_cur = intx4{4 * g, 4 * g + 1, 4 * g + 2, 4 * g + 3};
    auto load_rows = [&](int w) __attribute__((always_inline)) {
        rows_cur = *reinterpret_cast<const intx4*>(p.perm_pad + (size_t)w * 16 + 4 * g);
    };
    float* const out_base = partial ? p.ws + (size_t)(-w_end_raw - 1) * 16 * (size_t)N : p.C;

    auto flush = [&]() __attribute__((always_inline)) {  // store the accumulators to rows_cur and clear them
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = rows_cur[r];
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                if (row < 0 || !act[s]) continue;
                if (c16 && !partial) {  // rounded to nearest even; a lane's FPL values are contiguous
                    uint16_t* dst16 = reinterpret_cast<uint16_t*>(p.C) + (size_t)row * (size_t)N + f0 + s * SW;
                    uint32_t pk[(FPL + 1) / 2];
#pragma unroll
                    for (int m = 0; m < FPL; m += 2) {
                        pk[m >> 1] = narrow16<BF16>(acc[s][m][r]);
                        if constexpr (FPL > 1) pk[m >> 1] |= narrow16<BF16>(acc[s][m + 1][r]) << 16;
                    }
                    if constexpr (FPL == 8) *reinterpret_cast<uintx4*>(dst16) = uintx4{pk[0], pk[1], pk[2], pk[3]};
                    else if constexpr (FPL == 4) *reinterpret_cast<uintx2*>(dst16) = uintx2{pk[0], pk[1]};
                    else if constexpr (FPL == 2) *reinterpret_cast<uint32_t*>(dst16) = pk[0];
                    else *dst16 = (uint16_t)pk[0];
                    continue;
                }
                float* dst = out_base + (size_t)row * (size_t)N + f0 + s * SW;
                if constexpr (FPL >= 4) {
#pragma unroll
                    for (int m = 0; m < FPL; m += 4) {
                        floatx4 v{acc[s][m][r], acc[s][m + 1][r], acc[s][m + 2][r], acc[s][m + 3][r]};
                        if (nt) __builtin_nontemporal_store(v, reinterpret_cast<floatx4*>(dst + m));
                        else *reinterpret_cast<floatx4*>(dst + m) = v;
                    }
                } else {
#pragma unroll
                    for (int m = 0; m < FPL; ++m) {
                        if (nt) __builtin_nontemporal_store(acc[s][m][r], dst + m);
                        else dst[m] = acc[s][m][r];
                    }
                }
            }
        }
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int m = 0; m < FPL; ++m) acc[s][m] = floatx4{0.f, 0.f, 0.f, 0.f};
    };

    auto load_meta = [&](int t, TileMeta<TW32>& m) __attribute__((always_inline)) {
        t = t < te ? t : te - 1;  // past the end: re-read the last tile (always in bounds)
        if constexpr (TW32) {
            m.cols = *reinterpret_cast<const intx4*>(p.a2b + (size_t)t * 32 + 8 * g);
            m.cols2 = *reinterpret_cast<const intx4*>(p.a2b + (size_t)t * 32 + 8 * g + 4);
            m.rowbits = reinterpret_cast<const uint32_t*>(p.bits)[(size_t)t * 16 + c];
        } else {
            m.cols = *reinterpret_cast<const intx4*>(p.a2b + (size_t)t * 16 + 4 * g);
            const uint64_t* bm = p.bits + (size_t)t * 4;
            m.bm[0] = bm[0]; m.bm[1] = bm[1]; m.bm[2] = bm[2]; m.bm[3] = bm[3];
        }
        m.tco = p.tco[t];
    };

    // 64-bit addressing: this lane's byte address of feature f0 in row 0 of either matrix, and the row pitch
    const uint64_t hot_base = reinterpret_cast<uint64_t>(g_Bhot) + (uint64_t)f0 * 2;
    const uint64_t cold_base = reinterpret_cast<uint64_t>(p.B) + (uint64_t)f0 * 2;
    const uint32_t row_bytes = (uint32_t)N * 2u;
    auto issue = [&](const TileMeta<TW32>& m, TileData<FPL, NS, QR>& d, int slot) __attribute__((always_inline)) {
        int32_t entry[QR];
        entry[0] = m.cols[0]; entry[1] = m.cols[1]; entry[2] = m.cols[2]; entry[3] = m.cols[3];
        if constexpr (TW32) { entry[4] = m.cols2[0]; entry[5] = m.cols2[1]; entry[6] = m.cols2[2]; entry[7] = m.cols2[3]; }
#pragma unroll
        for (int q = 0; q < QR; ++q) {
            if constexpr (LDS) {
                // the lane's address as in the register form; the data lands in LDS
                uint64_t row;
                if constexpr (ADDR == kAddrNarrow) {
                    row = cold_base + (uint64_t)((__umul24((uint32_t)entry[q], (uint32_t)N)) << 1);
                } else {
                    const int32_t e = entry[q];
                    const bool hot = ADDR == kAddrHot && e < 0;
                    row = (uint64_t)(uint32_t)(hot ? ~e : e) * (uint64_t)row_bytes + (hot ? hot_base : cold_base);
                }
                uint32_t* const plane = stage_wave + (slot * 4 + q) * DW * 64;
                if constexpr (FPL == 8) {
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(row),
                                                     (__attribute__((address_space(3))) void*)(plane), 16, 0, 0);
                } else {
#pragma unroll
                    for (int k = 0; k < DW; ++k)
                        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(row + 4u * k),
                                                         (__attribute__((address_space(3))) void*)(plane + k * 64), 4, 0, 0);
                }
            } else if constexpr (ADDR == kAddrNarrow) {
                const uint32_t off = (__umul24((uint32_t)entry[q], (uint32_t)N) + (uint32_t)f0) << 1;
                const uint16_t* row = reinterpret_cast<const uint16_t*>(reinterpret_cast<const char*>(p.B) + (size_t)off);
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    if constexpr (TAIL) {
#pragma unroll
                        for (int k = 0; k < Chunk<FPL>::DW; ++k) d.b[s][q].d[k] = 0;
                        if (act[s]) load_chunk<FPL>(row + s * SW, d.b[s][q]);
                    } else {
                        load_chunk<FPL>(row + s * SW, d.b[s][q]);
                    }
                }
            } else {
                // one 32x32+64-bit multiply-add on top of the lane's precomputed base(s)
                const int32_t e = entry[q];
                const bool hot = ADDR == kAddrHot && e < 0;
                const uint64_t row = (uint64_t)(uint32_t)(hot ? ~e : e) * (uint64_t)row_bytes + (hot ? hot_base : cold_base);
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    if constexpr (TAIL) {
#pragma unroll
                        for (int k = 0; k < Chunk<FPL>::DW; ++k) d.b[s][q].d[k] = 0;
                        if (act[s]) load_chunk_global<FPL>(row + (uint64_t)(s * SW * 2), d.b[s][q]);
                    } else {
                        load_chunk_global<FPL>(row + (uint64_t)(s * SW * 2), d.b[s][q]);
                    }
                }
            }
        }
        uint32_t nib, i0, tile_cnt = 0;   // tile_cnt: entries of the tile (cooperative fetch only)
        if constexpr (TW32) {
            // the row's entries before this lane's byte, and the entries of the rows above by an inclusive
            // prefix sum of the rows' counts over the sixteen lanes of the group (DPP row shifts; a lane that
            // would read from outside its row adds zero)
            const uint32_t rb = m.rowbits;
            const uint32_t cnt = (uint32_t)__builtin_popcount(rb);
            uint32_t incl = cnt;
            incl += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)incl, 0x111, 0xf, 0xf, true);   // row_shr:1
            incl += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)incl, 0x112, 0xf, 0xf, true);   // row_shr:2
            incl += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)incl, 0x114, 0xf, 0xf, true);   // row_shr:4
            incl += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)incl, 0x118, 0xf, 0xf, true);   // row_shr:8
            nib = (rb >> (8 * g)) & 255u;
            i0 = (uint32_t)m.tco + (incl - cnt) + (uint32_t)__builtin_popcount(rb & ((1u << (8 * g)) - 1u));
        } else {
            // this lane's bitmap word and the popcount of the words below it, by plain selects
            const int c0 = __builtin_popcountll(m.bm[0]), c1 = __builtin_popcountll(m.bm[1]),
                      c2 = __builtin_popcountll(m.bm[2]);
            uint64_t word = m.bm[0];
            word = w1 ? m.bm[1] : word;
            word = w2 ? m.bm[2] : word;
            word = w3 ? m.bm[3] : word;
            const int pre = (w1 ? c0 : 0) + (w2 ? c1 : 0) + (w3 ? c2 : 0);
            nib = (uint32_t)(word >> sh) & 15u;
            i0 = (uint32_t)(m.tco + pre + __builtin_popcountll(word & below_mask));
            if constexpr (COOP) tile_cnt = (uint32_t)(c0 + c1 + c2 + __builtin_popcountll(m.bm[3]));
        }
        if constexpr (COOP) {
            const uint32_t cnt = tile_cnt;
            const uint32_t first_half = (uint32_t)m.tco & ~1u;        // first loaded value (dword aligned)
            const uint32_t span = ((uint32_t)m.tco & 1u) + cnt;       // halves from there to the tile's end
            const uint32_t nchunk = (span + 127u) >> 7;               // 0..3
            const uint32_t* v32 = reinterpret_cast<const uint32_t*>(p.vals) + (first_half >> 1);
            d.v[0] = 0; d.v[1] = 0; d.v[2] = 0;
            // only the lanes whose dword holds values of this tile read (so nothing is read past the tile)
            if ((uint32_t)lane * 2u < span) d.v[0] = v32[lane];
            if (nchunk > 1 && (uint32_t)(64 + lane) * 2u < span) d.v[1] = v32[64 + lane];
            if (nchunk > 2 && (uint32_t)(128 + lane) * 2u < span) d.v[2] = v32[128 + lane];
            d.v[3] = i0 - first_half;
            d.nchunk = nchunk;
        } else if constexpr (SPAN) {
            // the three dwords that hold values i0 .. i0+3, and the shift that brings value i0 to bit 0
            struct __attribute__((aligned(4))) Span { uint32_t a, b, c; };
            const Span sp = *reinterpret_cast<const Span*>(reinterpret_cast<const char*>(p.vals) + (size_t)(uint32_t)((i0 & ~1u) << 1));
            d.v[0] = sp.a; d.v[1] = sp.b; d.v[2] = sp.c; d.v[3] = (i0 & 1u) << 4;
            if constexpr (TW32) {   // the values of the upper nibble follow those of the lower one
                const uint32_t i1 = i0 + (uint32_t)__builtin_popcount(nib & 15u);
                const Span sq = *reinterpret_cast<const Span*>(reinterpret_cast<const char*>(p.vals) + (size_t)(uint32_t)((i1 & ~1u) << 1));
                d.v[4] = sq.a; d.v[5] = sq.b; d.v[6] = sq.c; d.v[7] = (i1 & 1u) << 4;
            }
            d.nchunk = 0;
        } else {
            const uint32_t i1 = i0 + (nib & 1u);
            const uint32_t i2 = i1 + ((nib >> 1) & 1u);
            const uint32_t i3 = i2 + ((nib >> 2) & 1u);
            const char* vb = reinterpret_cast<const char*>(p.vals);
            d.v[0] = *reinterpret_cast<const uint16_t*>(vb + (size_t)(uint32_t)(i0 << 1));
            d.v[1] = *reinterpret_cast<const uint16_t*>(vb + (size_t)(uint32_t)(i1 << 1));
            d.v[2] = *reinterpret_cast<const uint16_t*>(vb + (size_t)(uint32_t)(i2 << 1));
            d.v[3] = *reinterpret_cast<const uint16_t*>(vb + (size_t)(uint32_t)(i3 << 1));
            d.nchunk = 0;
        }
        d.nib = nib;
    };

    // LDS staging: the B rows of the tile in ring slot `slot`, which the wait above this call has
    // seen arrive, from LDS into the registers the multiply reads
    auto fetch_staged = [&](TileData<FPL, NS, QR>& d, int slot) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t* plane = stage_wave + (slot * 4 + q) * DW * 64;
            if constexpr (FPL == 8) {
                const uintx4 v = *reinterpret_cast<const uintx4*>(plane + lane * 4);
                d.b[0][q].d[0] = v.x; d.b[0][q].d[1] = v.y; d.b[0][q].d[2] = v.z; d.b[0][q].d[3] = v.w;
            } else {
#pragma unroll
                for (int k = 0; k < DW; ++k) d.b[0][q].d[k] = plane[k * 64 + lane];
            }
        }
    };

    // The sparse tile as this lane's MFMA operand: four fp16 values (zero where the bit is clear).
    auto operand_a = [&](const TileData<FPL, NS, QR>& d) __attribute__((always_inline)) {
        const uint32_t nib = d.nib;
        if constexpr (TW32) {
            // eight positions: the lower nibble takes its halves from v[0..3], the upper one from v[4..7]
            uintx4 a;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t lo = __builtin_amdgcn_alignbit(d.v[4 * h + 1], d.v[4 * h], d.v[4 * h + 3]);
                const uint32_t hi = __builtin_amdgcn_alignbit(d.v[4 * h + 2], d.v[4 * h + 1], d.v[4 * h + 3]);
                const int at = (int)(((nib >> (4 * h)) & 15u) << 2);
                const uint32_t s_lo = (uint32_t)__builtin_amdgcn_ds_bpermute(at, (int)lut_lo);
                const uint32_t s_hi = (uint32_t)__builtin_amdgcn_ds_bpermute(at, (int)lut_hi);
                a[2 * h] = __builtin_amdgcn_perm(hi, lo, s_lo);
                a[2 * h + 1] = __builtin_amdgcn_perm(hi, lo, s_hi);
            }
            return a;
        } else
        if constexpr (COOP) {
            // This lane's values are halves r0..r0+3 of what the wave loaded (r0 = d.v[3]): they lie in
            // the dwords j, j+1, j+2 with j = r0 >> 1, each held by lane (dword & 63) of chunk
            // (dword >> 6).  Fetch the three, shift them down by the odd half, and route half k to the
            // k-th set bit of nib (zero to the clear bits) with two byte permutes whose selectors come
            // from a 16-entry table that lanes 0..15 hold.
            const uint32_t r0 = d.v[3];
            const uint32_t j = r0 >> 1;
            const int nchunk = __builtin_amdgcn_readfirstlane((int)d.nchunk);
            uint32_t w[3];
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                const uint32_t dw = j + (uint32_t)k;
                const int addr = (int)(dw << 2);  // source lane * 4; the hardware uses it modulo 64 lanes
                uint32_t x = (uint32_t)__builtin_amdgcn_ds_bpermute(addr, (int)d.v[0]);
                if (nchunk > 1) {
                    const uint32_t x1 = (uint32_t)__builtin_amdgcn_ds_bpermute(addr, (int)d.v[1]);
                    x = ((dw >> 6) == 1u) ? x1 : x;
                }
                if (nchunk > 2) {
                    const uint32_t x2 = (uint32_t)__builtin_amdgcn_ds_bpermute(addr, (int)d.v[2]);
                    x = ((dw >> 6) == 2u) ? x2 : x;
                }
                w[k] = x;
            }
            const uint32_t sh = (r0 & 1u) << 4;
            const uint32_t lo = __builtin_amdgcn_alignbit(w[1], w[0], sh);  // halves r0, r0+1
            const uint32_t hi = __builtin_amdgcn_alignbit(w[2], w[1], sh);  // halves r0+2, r0+3
            const int at = (int)(nib << 2);
            const uint32_t s_lo = (uint32_t)__builtin_amdgcn_ds_bpermute(at, (int)lut_lo);
            const uint32_t s_hi = (uint32_t)__builtin_amdgcn_ds_bpermute(at, (int)lut_hi);
            return uintx2{__builtin_amdgcn_perm(hi, lo, s_lo), __builtin_amdgcn_perm(hi, lo, s_hi)};
        } else if constexpr (SPAN) {
            // d.v[0..2] hold the lane's four consecutive values from bit d.v[3] on; half k goes to the k-th set bit of nib
            const int at = (int)(nib << 2);
            const uint32_t s_lo = (uint32_t)__builtin_amdgcn_ds_bpermute(at, (int)lut_lo);
            const uint32_t s_hi = (uint32_t)__builtin_amdgcn_ds_bpermute(at, (int)lut_hi);
            const uint32_t lo = __builtin_amdgcn_alignbit(d.v[1], d.v[0], d.v[3]);
            const uint32_t hi = __builtin_amdgcn_alignbit(d.v[2], d.v[1], d.v[3]);
            return uintx2{__builtin_amdgcn_perm(hi, lo, s_lo), __builtin_amdgcn_perm(hi, lo, s_hi)};
        } else {
            const uint32_t a0 = (nib & 1u) ? d.v[0] : 0u;
            const uint32_t a1 = (nib & 2u) ? d.v[1] : 0u;
            const uint32_t a2 = (nib & 4u) ? d.v[2] : 0u;
            const uint32_t a3 = (nib & 8u) ? d.v[3] : 0u;
            return uintx2{a0 | (a1 << 16), a2 | (a3 << 16)};
        }
    };
    using OperandA = std::conditional_t<TW32, uintx4, uintx2>;

    auto multiply = [&](const TileData<FPL, NS, QR>& d, const OperandA au) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int m = 0; m < FPL; ++m) {
                const uint32_t sel = (m & 1) ? 0x07060302u : 0x05040100u;
                if constexpr (TW32) {
                    const uintx4 bu{__builtin_amdgcn_perm(d.b[s][1].d[m >> 1], d.b[s][0].d[m >> 1], sel),
                                    __builtin_amdgcn_perm(d.b[s][3].d[m >> 1], d.b[s][2].d[m >> 1], sel),
                                    __builtin_amdgcn_perm(d.b[s][5].d[m >> 1], d.b[s][4].d[m >> 1], sel),
                                    __builtin_amdgcn_perm(d.b[s][7].d[m >> 1], d.b[s][6].d[m >> 1], sel)};
                    if constexpr (BF16)
                        acc[s][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bfloat8, au),
                                                                            __builtin_bit_cast(bfloat8, bu), acc[s][m], 0, 0, 0);
                    else
                        acc[s][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, au),
                                                                           __builtin_bit_cast(half8, bu), acc[s][m], 0, 0, 0);
                } else {
                    const uintx2 bu{__builtin_amdgcn_perm(d.b[s][1].d[m >> 1], d.b[s][0].d[m >> 1], sel),
                                    __builtin_amdgcn_perm(d.b[s][3].d[m >> 1], d.b[s][2].d[m >> 1], sel)};
                    if constexpr (BF16)
                        acc[s][m] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(shortx4, au),
                                                                              __builtin_bit_cast(shortx4, bu), acc[s][m], 0, 0, 0);
                    else
                        acc[s][m] = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(half4, au),
                                                                          __builtin_bit_cast(half4, bu), acc[s][m], 0, 0, 0);
                }
            }
    };

    // window bookkeeping (all wave-uniform): w is the window being accumulated, wend its
    // one-past-last tile, wend_next that of window w+1 (requested one window ahead)
    int w = w_begin;
    int wend = partial ? te : p.rwo[w + 1];
    int wend_next = partial ? te : p.rwo[(w + 2 < w_end) ? w + 2 : w_end];
    auto next_window = [&]() __attribute__((always_inline)) {
        ++w;
        wend = wend_next;
        if (w < w_end) {
            load_rows(w);
            wend_next = p.rwo[(w + 2 < w_end) ? w + 2 : w_end];
        }
    };
    if (!partial) {
        load_rows(w);
        while (w < w_end && wend == tb) {  // leading empty windows: rows of zeros
            flush();
            next_window();
        }
    }
    if (tb >= te) return;

    auto after_tile = [&](int tt) __attribute__((always_inline)) {  // tile tt has been multiplied: close the window(s) ending there
        if (__builtin_expect(tt + 1 != wend, 1)) return;
        flush();
        if (partial) return;
        next_window();
        while (w < w_end && wend == tt + 1) {  // empty windows inside the run
            flush();
            next_window();
        }
    };

    if constexpr (DEPTH == 0) {
        // ablation: every tile's loads are issued only when the tile is computed
        TileMeta<TW32> m;
        TileData<FPL, NS, QR> d;
        for (int tt = tb; tt < te; ++tt) {
            load_meta(tt, m);
            issue(m, d, 0);
            multiply(d, operand_a(d));
            after_tile(tt);
        }
    } else {
        // Ring of R = DEPTH+1 buffers; tile x uses slot (x - tb) % R, for its data and, before
        // that, for its index words.  vmcnt retires loads in issue order: using the column ids of a
        // tile waits for every load issued before them.  They are therefore requested DEPTH+1 tiles
        // before the rows they address (tile tt+2*DEPTH+1 while tile tt is multiplied), so that the
        // wait leaves the rows of the DEPTH tiles issued since then in flight.
        TileMeta<TW32> meta[R];
        TileData<FPL, NS, QR> data[R];
#pragma unroll
        for (int r = 0; r < R; ++r) load_meta(tb + r, meta[r]);
#pragma unroll
        for (int r = 0; r < DEPTH; ++r) {
            issue(meta[r], data[r], r);
            load_meta(tb + R + r, meta[r]);
        }
        for (int t = tb; t < te; t += R) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int tt = t + r;
                if (tt >= te) break;
                // tile tt's sparse operand first: its cross-lane fetch (if any) shares a wait counter
                // with the scalar index loads issued next
                if constexpr (LDS) {
                    // everything requested so far (this tile's rows among it) has arrived; the next
                    // tile's requests follow only after the read-back, so they stay in flight during
                    // the multiply.  vmcnt(0), other counters untouched.
                    __builtin_amdgcn_sched_barrier(0);
                    __builtin_amdgcn_s_waitcnt(0x0F70);
                    fetch_staged(data[r], r);
                    __builtin_amdgcn_sched_barrier(0);
                }
                const OperandA au = operand_a(data[r]);
                if constexpr (FETCH != kFetchLane) __builtin_amdgcn_sched_barrier(0);
                const int s = (r + DEPTH) % R;            // slot of tile tt+DEPTH
                issue(meta[s], data[s], s);
                load_meta(tt + 2 * DEPTH + 1, meta[s]);   // the slot's next tile
                multiply(data[r], au);
                after_tile(tt);
            }
        }
    }
}

template <int FPL, int NS, int DEPTH, int ADDR, int FETCH, bool TAIL, bool BF16>
void launch_one(const ExecParams& p, hipStream_t stream) {
    const int blocks = ((p.n_blocks + 7) / 8) * 8;
    dim3 grid(blocks, p.grid_y), block(kWavesPerBlock * 64);
    if constexpr (DEPTH == 1 && NS == 1 && !TAIL && !BF16 && FPL >= 2) {
        if (p.lds) {
            hipLaunchKernelGGL((spmm_tiles_kernel<FPL, NS, DEPTH, ADDR, FETCH, TAIL, BF16, true>), grid, block, 0, stream, p.rwo,
                               p.tco, p.a2b, p.bits, p.vals, p.perm_pad, p.items, p.B, p.B_hot, p.C, p.ws, p.n_items,
                               p.n_blocks, p.N, p.store_mode);
            return;
        }
    }
    if constexpr (FETCH == kFetchSpan && (DEPTH == 1 || DEPTH == 2)) {
        if (p.tw32) {
            hipLaunchKernelGGL((spmm_tiles_kernel<FPL, NS, DEPTH, ADDR, FETCH, TAIL, BF16, false, true>), grid, block, 0, stream,
                               p.rwo, p.tco, p.a2b, p.bits, p.vals, p.perm_pad, p.items, p.B, p.B_hot, p.C, p.ws, p.n_items,
                               p.n_blocks, p.N, p.store_mode);
            return;
        }
    }
    hipLaunchKernelGGL((spmm_tiles_kernel<FPL, NS, DEPTH, ADDR, FETCH, TAIL, BF16>), grid, block, 0, stream, p.rwo, p.tco, p.a2b,
                       p.bits, p.vals, p.perm_pad, p.items, p.B, p.B_hot, p.C, p.ws, p.n_items, p.n_blocks, p.N,
                       p.store_mode);
}

template <int FPL, int NS, int DEPTH, int ADDR, bool TAIL, bool BF16>
void launch_fetch(const ExecParams& p, hipStream_t stream) {
    switch (p.fetch) {
        case kFetchCoop: launch_one<FPL, NS, DEPTH, ADDR, kFetchCoop, TAIL, BF16>(p, stream); break;
        case kFetchSpan: launch_one<FPL, NS, DEPTH, ADDR, kFetchSpan, TAIL, BF16>(p, stream); break;
        default: launch_one<FPL, NS, DEPTH, ADDR, kFetchLane, TAIL, BF16>(p, stream); break;
    }
}

template <int FPL, int NS, int DEPTH, bool TAIL, bool BF16>
void launch_type(const ExecParams& p, hipStream_t stream) {
    switch (p.addr) {
        case kAddrHot: launch_fetch<FPL, NS, DEPTH, kAddrHot, TAIL, BF16>(p, stream); break;
        case kAddrWide: launch_fetch<FPL, NS, DEPTH, kAddrWide, TAIL, BF16>(p, stream); break;
        default: launch_fetch<FPL, NS, DEPTH, kAddrNarrow, TAIL, BF16>(p, stream); break;
    }
}

template <int FPL, int NS, int DEPTH, bool TAIL>
void launch_depth(const ExecParams& p, hipStream_t stream) {
    launch_type<FPL, NS, DEPTH, TAIL, ACC_TILE_BF16 != 0>(p, stream);
}

template <int FPL, int NS, bool TAIL>
void launch_variant(const ExecParams& p, hipStream_t stream) {
    switch (p.depth) {
        case 0: launch_depth<FPL, NS, 0, TAIL>(p, stream); break;
        case 1: launch_depth<FPL, NS, 1, TAIL>(p, stream); break;
        case 3: launch_depth<FPL, NS, 3, TAIL>(p, stream); break;
        default: launch_depth<FPL, NS, 2, TAIL>(p, stream); break;
    }
}

// Without a tail only the slab shapes that a power-of-two or 128-multiple N produces exist.
template <int FPL>
void launch_shape(const ExecParams& p, hipStream_t stream) {
    if (p.tail) {
        if (p.ns == 2) launch_variant<FPL, 2, true>(p, stream);
        else launch_variant<FPL, 1, true>(p, stream);
    } else {
        if constexpr (FPL == 8) {
            if (p.ns == 2) { launch_variant<8, 2, false>(p, stream); return; }
        }
        launch_variant<FPL, 1, false>(p, stream);
    }
}

}  // namespace

#define ACC_TILE_LAUNCHER_NAME2(FPL, T) launch_tiles_f##FPL##_t##T
#define ACC_TILE_LAUNCHER_NAME(FPL, T) ACC_TILE_LAUNCHER_NAME2(FPL, T)
void ACC_TILE_LAUNCHER_NAME(ACC_TILE_FPL, ACC_TILE_BF16)(const ExecParams& p, hipStream_t stream) {
    launch_shape<ACC_TILE_FPL>(p, stream);
}

}  // namespace accspmm
