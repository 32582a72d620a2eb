// Copy -> copy chain: the smallest pair of dependent tiled kernels, used to measure what the
// synchronisation itself costs (the paper's overhead experiment, Section V: tile i of the
// consumer depends on tile i of the producer, and the kernels do nothing but move bytes).
// Stage 0 copies src to mid, stage 1 copies mid to dst; a tile is a contiguous run of 16-byte
// units.  Dispatch, post and wait are the ones the GeMM and conv chains use.
#include <hip/hip_runtime.h>
#include "chain_args.h"
#include "launch.h"
#include "sync_device.hpp"

namespace depsync {

typedef uint32_t copy_u32x4 __attribute__((ext_vector_type(4)));

// StageDesc fields of a copy stage: A source, C destination, N total 16-byte units, K units
// per tile, grid_x tiles, grid_y = 1.
template <bool SYNC, class DR>
__device__ __forceinline__ void copy_tile(const ChainArgs& args, const StageDesc& s, uint32_t tx, uint32_t rel,
                                          uint64_t t_enter, DR& dr) {
    const uint32_t tid = threadIdx.x;
    WaitCtx wctx{&args, rel, true};
    const bool tracing = SYNC && (args.flags & DS_FLAG_TRACE) && args.trace != nullptr && rel < args.trace_cap;
    uint64_t t_start = 0, t_ready = 0;
    if (tracing) t_start = now_ticks();

    if constexpr (SYNC) {
        if (s.dep_kind != DEP_NONE) {
            // TileSync: the producer's tile of the same index; RowSync: one semaphore that all
            // producer tiles post to (the consumer then starts when the whole stage is done)
            const uint32_t* sem = s.sems + policy_sem(s.dep_kind, tx, 0, s.prod_grid_y, s.stride) * SYNC_WORD_STRIDE;
            const uint32_t target = s.sem_target_base + s.sem_value;
            const uint32_t first = sem_load(sem);
            const bool polled = !sem_reached(first, target);
            sem_wait(wctx, sem, target, first);
            count_wait(args, polled);
        }
    }
    if (tracing) t_ready = now_ticks();

    const uint64_t u0 = (uint64_t)tx * s.K;
    const uint64_t left = (uint64_t)s.N - u0;
    const uint32_t n = left < (uint64_t)s.K ? (uint32_t)left : s.K;
    const copy_u32x4* src = static_cast<const copy_u32x4*>(s.A) + u0;
    copy_u32x4* dst = static_cast<copy_u32x4*>(s.C) + u0;
    const bool through = SYNC && s.post_kind != DEP_NONE;   // a tile that posts writes through to memory
    dr.peek();
    if (wctx.ok) {
        uint32_t i = tid;
        for (; i + 3 * 256 < n; i += 4 * 256) {             // four 16-byte loads in flight per lane
            const copy_u32x4 v0 = src[i], v1 = src[i + 256], v2 = src[i + 512], v3 = src[i + 768];
            if (through) {
                asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(dst + i), "v"(v0) : "memory");
                asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(dst + i + 256), "v"(v1) : "memory");
                asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(dst + i + 512), "v"(v2) : "memory");
                asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(dst + i + 768), "v"(v3) : "memory");
            } else {
                dst[i] = v0; dst[i + 256] = v1; dst[i + 512] = v2; dst[i + 768] = v3;
            }
        }
        for (; i < n; i += 256) {
            const copy_u32x4 v = src[i];
            if (through) asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(dst + i), "v"(v) : "memory");
            else dst[i] = v;
        }
    }
    dr.grab();
    if constexpr (SYNC) post_tile<true>(args, s, tx, tx, 0);
    if (tracing && tid == 0) {
        TraceRec r;
        r.rel = rel; r.where = hw_where(s.dep_kind != DEP_NONE ? 1u : 0u); r.tx = tx; r.ty = 0;
        r.t_enter = t_enter; r.t_start = t_start; r.t_ready = t_ready; r.t_end = now_ticks();
        args.trace[rel] = r;
    }
}

template <bool SYNC>
__global__ __launch_bounds__(256, 8) void copy_chain_kernel(const ChainArgs args) {
    __shared__ uint32_t slot[4];
    if constexpr (!SYNC) {
        NoDrawer nd;
        const TileId t = hw_order_tile(args);
        copy_tile<false>(args, args.st[t.stage], t.tx, t.rel, 0, nd);
    } else {
        Drawer dr(args, slot);
        const bool hw_order = (args.flags & DS_FLAG_HW_ORDER) != 0;
        if (hw_order) dr.open = args.stage_hi + 1;
        for (;;) {
            uint64_t t_enter = 0;
            if (args.flags & DS_FLAG_TRACE) t_enter = now_ticks();
            const TileId t = hw_order ? hw_order_tile(args) : dr.next();
            if (t.rel == 0xffffffffu) return;
            copy_tile<true>(args, args.st[t.stage], t.tx, t.rel, t_enter, dr);
            if (hw_order) return;
        }
    }
}

hipError_t launch_copy(bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a) {
    if (sync) hipLaunchKernelGGL(copy_chain_kernel<true>, dim3(n_blocks), dim3(256), 0, stream, a);
    else hipLaunchKernelGGL(copy_chain_kernel<false>, dim3(n_blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace depsync
