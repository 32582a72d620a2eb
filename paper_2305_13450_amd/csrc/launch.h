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

// nullptr for ids outside [1, 13].
const TileShape* tile_shape(int tile);

// Launch n_blocks workgroups of the chain kernel for macro-tile `tile`, element type `dtype`
// (0 = bf16, 1 = fp16) and A addressing mode `amode`, with the synchronisation hooks compiled
// in or out.
hipError_t launch_chain_kernel(int tile, int dtype, uint32_t amode, bool sync, uint32_t n_blocks,
                               hipStream_t stream, const ChainArgs& a);

hipError_t launch_fill_u32(uint32_t* p, uint32_t value, uint32_t n, hipStream_t stream);

// The wait kernel of Section III-B: one wave that ends when `want` tiles of stage `stage` have been
// drawn from the chain's dispatch queues (i.e. the producer launch, on another stream, holds its
// workgroup slots), or when the chain's spin limit expires (counted as a time-out in the status
// block).  Launches queued behind it on `stream` start after that.
hipError_t launch_wait_draws(const ChainArgs& a, uint32_t stage, uint32_t want, hipStream_t stream);

// Register-only MFMA loop: n_blocks workgroups of 256 threads, 8 * iters MFMAs (32x32x16 bf16)
// per wave; src holds 1 MiB of operand bits, out n_blocks * 256 floats (practically never written).
hipError_t launch_mfma_calibration(const void* src, float* out, int n_blocks, int iters, hipStream_t stream);

// One family per translation unit (kern_*.hip).
hipError_t launch_bf16_gemm(int tile, bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a);
hipError_t launch_f16_gemm(int tile, bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a);
hipError_t launch_bf16_conv(int tile, bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a);
hipError_t launch_f16_conv(int tile, bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a);
hipError_t launch_bf16_gemm_gen(int tile, bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a);
hipError_t launch_f16_gemm_gen(int tile, bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a);
hipError_t launch_bf16_gemm_attn(int tile, bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a);
hipError_t launch_f16_gemm_attn(int tile, bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a);
hipError_t launch_copy(bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a);   // kern_copy.hip

}  // namespace depsync
