// The chain kernel template and its per-(element type, A addressing mode) launcher.
//
// One kernel template serves every launch of a chain: a workgroup draws the stage and
// tile it runs from the chain's dispatch queues (see sync_device.hpp for why producer
// and consumer share one body).  It is instantiated per macro-tile shape, element type, A
// addressing mode, and with the synchronisation hooks compiled in (FINE, STREAMSYNC) or out
// (PLAIN).  The attention tiles live in instantiations of their own (MIDK: 0 no attention stage,
// 1 prompt-phase attention, 2 token generation), used only by chains that have such a stage, so
// that their registers do not weigh on the allocation of the kernels every other chain runs.  Each translation unit kern_*.hip instantiates one
// (type, mode) family so that the families compile in parallel.
#pragma once
#include <hip/hip_runtime.h>
#include "chain_args.h"
#include "attn_decode.hpp"
#include "attn_tile.hpp"
#include "gemm_tile.hpp"
#include "sync_device.hpp"

namespace depsync {

template <class Cfg, typename T, bool SYNC, uint32_t AMODE, int MIDK, class DR>
__device__ __forceinline__ void run_tile(const ChainArgs& args, const TileId t, char* lds, uint64_t t_enter, DR& dr) {
    const StageDesc& s = args.st[t.stage];
    if constexpr (AMODE == A_DENSE && MIDK != 0) {
        if (s.op == OP_ATTN) {   // middle stage of the attention chain
            if constexpr (MIDK == 2) attn_decode_tile<T, SYNC>(args, s, t.tx, t.ty, t.rel, lds, t_enter, dr);   // token generation (seq = 1)
            else attn_tile<T, SYNC>(args, s, t.tx, t.ty, t.rel, lds, t_enter, dr);
            return;
        }
    }
    if constexpr (SYNC) {
        // a dependent stage that is itself waited for exists only in chains of three or four
        // convolutions (the middle stage of a GeMM chain is the attention tile)
        constexpr bool MID = AMODE == A_CONV3X3;
        const bool posts = s.post_kind != DEP_NONE;
        if (s.dep_kind == DEP_ROW || s.dep_kind == DEP_CONV_ROW) {   // one wait, before the first slice
            if constexpr (MID) {
                if (posts) { gemm_tile<Cfg, T, true, AMODE, 1, true>(args, s, t.tx, t.ty, t.rel, lds, t_enter, dr); return; }
            }
            gemm_tile<Cfg, T, true, AMODE, 1, false>(args, s, t.tx, t.ty, t.rel, lds, t_enter, dr);
            return;
        }
        if (s.dep_kind != DEP_NONE) {                                // waits inside the K loop as well
            if constexpr (MID) {
                if (posts) { gemm_tile<Cfg, T, true, AMODE, 2, true>(args, s, t.tx, t.ty, t.rel, lds, t_enter, dr); return; }
            }
            gemm_tile<Cfg, T, true, AMODE, 2, false>(args, s, t.tx, t.ty, t.rel, lds, t_enter, dr);
            return;
        }
    }
    gemm_tile<Cfg, T, SYNC, AMODE, 0, SYNC>(args, s, t.tx, t.ty, t.rel, lds, t_enter, dr);
}

template <class Cfg, typename T, bool SYNC, uint32_t AMODE, int MIDK>
__global__ __launch_bounds__(256, Cfg::MINB) void chain_kernel(const ChainArgs args) {
    // One LDS object only: with a second one the compiler can no longer tell the DMA writes
    // into the idle stage from the fragment reads of the current stage and serialises them.
    static_assert(Cfg::LDS_BYTES >= ATT_LDS_BYTES, "the attention tile stages its K and V blocks in the same LDS");
    __shared__ __attribute__((aligned(1024))) char lds[Cfg::LDS_BYTES];

    if constexpr (!SYNC) {
        // hooks compiled out: one tile per workgroup, named by the hardware's block index
        NoDrawer nd;
        run_tile<Cfg, T, false, AMODE, MIDK>(args, hw_order_tile(args), lds, 0, nd);
    } else {
        Drawer dr(args, reinterpret_cast<uint32_t*>(lds));
        const bool hw_order = (args.flags & DS_FLAG_HW_ORDER) != 0;   // one tile, from the block index
        if (hw_order) dr.open = args.stage_hi + 1;                    // nothing to draw
        for (;;) {
            uint64_t t_enter = 0;
            if (args.flags & DS_FLAG_TRACE) t_enter = now_ticks();
            const TileId t = hw_order ? hw_order_tile(args) : dr.next();
            if (t.rel == 0xffffffffu) return;
            run_tile<Cfg, T, true, AMODE, MIDK>(args, t, lds, t_enter, dr);
            if (hw_order) return;
        }
    }
}

//                        TM   TN  WM WN  workgroups per CU, LDS stages of A (, of B if fewer)
using Cfg256x256 = TileCfg<256, 256, 2, 2, 1, 3, 2>;   // 96 + 64 KB: three stages of A, two of B
using Cfg256x128 = TileCfg<256, 128, 2, 2, 1, 3>;   // 144 KB
using Cfg128x256 = TileCfg<128, 256, 2, 2, 1, 3>;   // 144 KB
using Cfg128x128 = TileCfg<128, 128, 2, 2, 2, 2>;   // 2 x 64 KB
using Cfg64x128 = TileCfg<64, 128, 2, 2, 2, 3>;     // 2 x 72 KB
using Cfg64x64 = TileCfg<64, 64, 2, 2, 2, 4>;       // 2 x 64 KB
using Cfg256x192 = TileCfg<256, 192, 2, 2, 1, 3, 2>;   // 96 + 48 KB: three stages of A, two of B
using Cfg128x192 = TileCfg<128, 192, 2, 2, 2, 2>;   // 2 x 80 KB
using Cfg256x64 = TileCfg<256, 64, 4, 1, 2, 2>;     // 2 x 80 KB
using Cfg64x64Deep = TileCfg<64, 64, 2, 2, 1, 8>;   // 128 KB: seven K steps in flight
using Cfg64x192 = TileCfg<64, 192, 2, 2, 1, 4>;     // 128 KB: three K steps in flight
using Cfg128x192Deep = TileCfg<128, 192, 2, 2, 1, 4>;   // 160 KB: three K steps in flight
using Cfg128x128Deep = TileCfg<128, 128, 2, 2, 1, 4>;   // 128 KB: three K steps in flight

template <class Cfg, typename T, uint32_t AMODE, int MIDK>
static hipError_t launch_cfg(bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a) {
    if (sync)
        hipLaunchKernelGGL((chain_kernel<Cfg, T, true, AMODE, MIDK>), dim3(n_blocks), dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((chain_kernel<Cfg, T, false, AMODE, MIDK>), dim3(n_blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

template <typename T, uint32_t AMODE, int MIDK = 0>
static hipError_t launch_family(int tile, bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a) {
    switch (tile) {
        case 1: return launch_cfg<Cfg256x256, T, AMODE, MIDK>(sync, n_blocks, stream, a);
        case 2: return launch_cfg<Cfg256x128, T, AMODE, MIDK>(sync, n_blocks, stream, a);
        case 3: return launch_cfg<Cfg128x256, T, AMODE, MIDK>(sync, n_blocks, stream, a);
        case 4: return launch_cfg<Cfg128x128, T, AMODE, MIDK>(sync, n_blocks, stream, a);
        case 5: return launch_cfg<Cfg64x128, T, AMODE, MIDK>(sync, n_blocks, stream, a);
        case 6: return launch_cfg<Cfg64x64, T, AMODE, MIDK>(sync, n_blocks, stream, a);
        case 7: return launch_cfg<Cfg256x192, T, AMODE, MIDK>(sync, n_blocks, stream, a);
        case 8: return launch_cfg<Cfg128x192, T, AMODE, MIDK>(sync, n_blocks, stream, a);
        case 9: return launch_cfg<Cfg256x64, T, AMODE, MIDK>(sync, n_blocks, stream, a);
        case 10: return launch_cfg<Cfg64x64Deep, T, AMODE, MIDK>(sync, n_blocks, stream, a);
        case 11: return launch_cfg<Cfg64x192, T, AMODE, MIDK>(sync, n_blocks, stream, a);
        case 12: return launch_cfg<Cfg128x192Deep, T, AMODE, MIDK>(sync, n_blocks, stream, a);
        case 13: return launch_cfg<Cfg128x128Deep, T, AMODE, MIDK>(sync, n_blocks, stream, a);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace depsync
