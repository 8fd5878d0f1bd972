// Shared between the tile-kernel translation units and the execute dispatcher.
#pragma once
#include "internal.h"

namespace accspmm {

constexpr int kWavesPerBlock = 4;   // wavefronts (work items) per thread block of the tile kernel
constexpr int kMaxN = 65536;
constexpr int kAddrNarrow = 0, kAddrWide = 1, kAddrHot = 2;   // how the tile kernel addresses rows of B
constexpr int kFetchLane = 0, kFetchCoop = 1, kFetchSpan = 2;   // how a tile's packed values reach the lanes
constexpr int kStoreStreaming = 1, kStoreNarrow = 2;           // bits of store_mode: nontemporal C stores; 16-bit C

struct ExecParams {
    const int32_t* __restrict__ rwo;
    const int32_t* __restrict__ tco;
    const int32_t* __restrict__ a2b;
    const uint64_t* __restrict__ bits;
    const uint16_t* __restrict__ vals;
    const int32_t* __restrict__ perm_pad;
    const WorkItem* __restrict__ items;
    const uint16_t* __restrict__ B;
    float* __restrict__ C;
    float* __restrict__ ws;
    int32_t n_items;
    int32_t n_blocks;  // logical thread blocks = ceil(n_items / kWavesPerBlock)
    int32_t N;
    int32_t addr;      // kAddrNarrow / kAddrWide / kAddrHot
    const uint16_t* __restrict__ B_hot;  // kAddrHot: the gathered most used rows of B
    int32_t fetch;     // kFetchLane / kFetchCoop / kFetchSpan
    bool tail;         // N is not a whole number of slabs
    bool bf16;         // values are bfloat16
    bool tw32;         // the plan's tiles are 16 x 32 (span fetch, depth 1 or 2)
    bool lds;          // B rows staged through an LDS double buffer instead of the register ring
    int32_t fpl, ns, grid_y, depth, store_mode;
};

// One function per (features per lane, value type); each lives in its own object file,
// compiled from tile_kernel.hip with ACC_TILE_FPL and ACC_TILE_BF16 defined.
#define ACC_DECLARE_TILE_LAUNCHER(FPL, T) void launch_tiles_f##FPL##_t##T(const ExecParams& p, hipStream_t stream);
ACC_DECLARE_TILE_LAUNCHER(1, 0) ACC_DECLARE_TILE_LAUNCHER(2, 0) ACC_DECLARE_TILE_LAUNCHER(4, 0) ACC_DECLARE_TILE_LAUNCHER(8, 0)
ACC_DECLARE_TILE_LAUNCHER(1, 1) ACC_DECLARE_TILE_LAUNCHER(2, 1) ACC_DECLARE_TILE_LAUNCHER(4, 1) ACC_DECLARE_TILE_LAUNCHER(8, 1)
#undef ACC_DECLARE_TILE_LAUNCHER

}  // namespace accspmm
