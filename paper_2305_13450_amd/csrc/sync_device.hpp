// Device side of the synchronisation subsystem: tile dispatch, post and wait
// (Sections III-B to III-D of the paper, re-thought for CDNA4).
//
//  * Dispatch.  The paper relies on CUDA issuing the blocks of the earlier-launched kernel
//    first and adds a one-thread "wait kernel" to order the launches (Section III-B).  HIP
//    makes no such promise across hardware queues, so here EVERY workgroup of every launch of
//    a chain draws a ticket from one shared counter and runs whatever tile the ticket names:
//    tickets [0,P) are producer tiles, [P,P+C) consumer tiles, in row-major order (Section
//    III-C).  A workgroup can only be spinning while it holds a ticket >= P, and by then all
//    tickets < P are held by resident workgroups that never wait, so every semaphore is
//    eventually posted whatever the dispatcher does.
//  * post: every wave makes its stores visible at agent scope, the workgroup meets at a
//    barrier, one lane does a release increment of the tile's semaphore (Section III-D).
//  * wait: every wave polls the same semaphore word (all lanes read one address, the result
//    is made scalar, so the spin loop is wave-uniform), sleeps between polls, and executes an
//    agent-scope acquire fence once the value is reached.  No lane-0 branch, no extra barrier.
#pragma once
#include <hip/hip_runtime.h>
#include "chain_args.h"

namespace depsync {

#define DS_FLAG_NO_REORDER 1u
#define DS_FLAG_COUNT 2u
#define DS_FLAG_REVERSE_ORDER 4u
#define DS_FLAG_HW_ORDER 8u

__device__ __forceinline__ uint32_t sem_load(const uint32_t* sem) {
    uint32_t v = __hip_atomic_load(sem, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return __builtin_amdgcn_readfirstlane(v);
}

__device__ __forceinline__ bool sem_reached(uint32_t v, uint32_t target) {
    return (int32_t)(v - target) >= 0;
}

__device__ __forceinline__ void acquire_agent() {
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

// State one wave keeps while it runs a tile.
struct WaitCtx {
    const ChainArgs* args;
    uint32_t ticket;     // relative ticket of the tile (for the status block)
    bool ok;             // false once a bounded wait expired: the tile's stores are skipped
};

__device__ __forceinline__ void note_timeout(WaitCtx& w) {
    w.ok = false;
    if ((threadIdx.x & 63) == 0) {
        StatusBlock* st = w.args->status;
        int prev = __hip_atomic_fetch_add(&st->timed_out, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (prev == 0)
            __hip_atomic_store(&st->first_timeout, (int32_t)w.ticket, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Block until *sem has reached target (or the spin limit expires).  Wave-uniform.
__device__ __forceinline__ void sem_wait(WaitCtx& w, const uint32_t* sem, uint32_t target, uint32_t first) {
    uint32_t v = first;
    const uint32_t limit = w.args->spin_limit;
    uint32_t spins = 0;
    while (!sem_reached(v, target)) {
        __builtin_amdgcn_s_sleep(4);
        v = sem_load(sem);
        if (limit != 0 && ++spins >= limit) {
            if (!sem_reached(v, target)) note_timeout(w);
            break;
        }
    }
}

__device__ __forceinline__ void count_wait(const ChainArgs& a, bool polled) {
    if ((a.flags & DS_FLAG_COUNT) && threadIdx.x == 0) {
        __hip_atomic_fetch_add(&a.status->waits, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (polled)
            __hip_atomic_fetch_add(&a.status->polling_waits, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Semaphore a producer tile (x,y) posts to / a consumer looks at, per policy (Fig. 4b):
//   row:     sem = y                      value = grid_x
//   tile:    sem = x*grid_y + y           value = 1
//   strided: sem = y*stride + x % stride  value = grid_x / stride
__device__ __forceinline__ uint32_t policy_sem(uint32_t kind, uint32_t x, uint32_t y, uint32_t grid_y, uint32_t stride) {
    switch (kind) {
        case DEP_TILE:
        case DEP_CONV_TILE:
            return x * grid_y + y;
        case DEP_STRIDED:
        case DEP_ATTN_QKV:
            return y * stride + (x % stride);
        default:
            return y;
    }
}

// post (Section III-D): called by all threads of the workgroup after the tile's stores.
__device__ __forceinline__ void post_tile(const ChainArgs& a, const StageDesc& s, uint32_t tile_lin, uint32_t x, uint32_t y) {
    if (s.post_kind == DEP_NONE) return;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __syncthreads();
    if (threadIdx.x == 0) {
        if (a.delay_tile == tile_lin + 1) {
            for (uint32_t i = 0; i < a.delay_iters; ++i) __builtin_amdgcn_s_sleep(127);
        }
        uint32_t idx = policy_sem(s.post_kind, x, y, s.grid_y, s.post_stride);
        __hip_atomic_fetch_add(&s.post_sems[idx], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        if (a.flags & DS_FLAG_COUNT)
            __hip_atomic_fetch_add(&a.status->posts, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Draw the tile this workgroup runs.  Returns the relative ticket in [0, total).
template <bool SYNC>
__device__ __forceinline__ uint32_t draw_ticket(const ChainArgs& a, uint32_t* lds_slot) {
    if (!SYNC || (a.flags & DS_FLAG_HW_ORDER)) return a.block_offset + blockIdx.x;
    if (threadIdx.x == 0) {
        uint32_t t = __hip_atomic_fetch_add(a.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *lds_slot = t - a.ticket_base;
    }
    __syncthreads();
    uint32_t t = *lds_slot;
    return __builtin_amdgcn_readfirstlane(t);
}

}  // namespace depsync
