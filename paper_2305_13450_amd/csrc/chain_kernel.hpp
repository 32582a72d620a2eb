// The chain kernel template and its per-(element type, A addressing mode) launcher.
//
// One kernel template serves every launch of a chain: a workgroup draws a ticket, finds the
// stage and tile the ticket names and runs that tile (see sync_device.hpp for why producer
// and consumer share one body).  It is instantiated per macro-tile shape, element type, A
// addressing mode, and with the synchronisation hooks compiled in (FINE, STREAMSYNC) or out
// (PLAIN).  Each translation unit kern_*.hip instantiates one (type, mode) family so that the
// families compile in parallel.
#pragma once
#include <hip/hip_runtime.h>
#include "chain_args.h"
#include "gemm_tile.hpp"
#include "sync_device.hpp"

namespace depsync {

template <class Cfg, typename T, bool SYNC, uint32_t AMODE>
__global__ __launch_bounds__(256, Cfg::MINB) void chain_kernel(const ChainArgs args) {
    __shared__ __attribute__((aligned(1024))) char lds[Cfg::LDS_BYTES];
    __shared__ uint32_t ticket_slot;

    const uint32_t rel = draw_ticket<SYNC>(args, &ticket_slot);
    uint32_t stage = 0;
    if (args.n_stages > 1 && rel >= args.first_ticket[1]) stage = 1;
    if (args.n_stages > 2 && rel >= args.first_ticket[2]) stage = 2;
    const StageDesc& s = args.st[stage];
    uint32_t tile_lin = rel - args.first_ticket[stage];
    if (SYNC && stage == 0 && (args.flags & DS_FLAG_REVERSE_ORDER))
        tile_lin = (args.first_ticket[1] - args.first_ticket[0]) - 1u - tile_lin;

    gemm_tile<Cfg, T, SYNC, AMODE>(args, s, tile_lin, rel, lds);
}

//                       TM   TN  WM WN  waves per SIMD
using Cfg256x256 = TileCfg<256, 256, 2, 2, 1>;
using Cfg256x128 = TileCfg<256, 128, 2, 2, 1>;
using Cfg128x256 = TileCfg<128, 256, 2, 2, 1>;
using Cfg128x128 = TileCfg<128, 128, 2, 2, 2>;
using Cfg64x128 = TileCfg<64, 128, 2, 2, 2>;
using Cfg64x64 = TileCfg<64, 64, 2, 2, 2>;

template <class Cfg, typename T, uint32_t AMODE>
static hipError_t launch_cfg(bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a) {
    if (sync)
        hipLaunchKernelGGL((chain_kernel<Cfg, T, true, AMODE>), dim3(n_blocks), dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((chain_kernel<Cfg, T, false, AMODE>), dim3(n_blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

template <typename T, uint32_t AMODE>
static hipError_t launch_family(int tile, bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a) {
    switch (tile) {
        case 1: return launch_cfg<Cfg256x256, T, AMODE>(sync, n_blocks, stream, a);
        case 2: return launch_cfg<Cfg256x128, T, AMODE>(sync, n_blocks, stream, a);
        case 3: return launch_cfg<Cfg128x256, T, AMODE>(sync, n_blocks, stream, a);
        case 4: return launch_cfg<Cfg128x128, T, AMODE>(sync, n_blocks, stream, a);
        case 5: return launch_cfg<Cfg64x128, T, AMODE>(sync, n_blocks, stream, a);
        case 6: return launch_cfg<Cfg64x64, T, AMODE>(sync, n_blocks, stream, a);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace depsync
