// Host-side interface between the C-ABI layer and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include "chain_args.h"

namespace depsync {

struct TileShape {
    int rows, cols;       // macro-tile
    int occupancy;        // workgroups resident per CU
    int wave_cols;        // columns of one wave's sub-tile (gate/up fusion needs a multiple of 64)
};

// nullptr for ids outside [1, 10].
const TileShape* tile_shape(int tile);

// Launch n_blocks workgroups of the chain kernel for macro-tile `tile`, element type `dtype`
// (0 = bf16, 1 = fp16) and A addressing mode `amode`, with the synchronisation hooks compiled
// in or out.
hipError_t launch_chain_kernel(int tile, int dtype, uint32_t amode, bool sync, uint32_t n_blocks,
                               hipStream_t stream, const ChainArgs& a);

hipError_t launch_fill_u32(uint32_t* p, uint32_t value, uint32_t n, hipStream_t stream);

// One family per translation unit (kern_*.hip).
hipError_t launch_bf16_gemm(int tile, bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a);
hipError_t launch_f16_gemm(int tile, bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a);
hipError_t launch_bf16_conv(int tile, bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a);
hipError_t launch_f16_conv(int tile, bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a);

}  // namespace depsync
