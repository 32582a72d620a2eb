// Device side of the synchronisation subsystem: tile dispatch, post and wait
// (Sections III-B to III-D of the paper, re-thought for CDNA4).
//
//  * Dispatch.  The paper relies on CUDA issuing the blocks of the earlier-launched kernel
//    first and adds a one-thread "wait kernel" to order the launches (Section III-B).  HIP
//    makes no such promise across hardware queues, so here the workgroups of every launch of
//    a chain draw their tiles from shared dispatch queues in which all producer tiles come
//    before the consumer tiles, each stage in row-major order (Section III-C); see Drawer.
//    A workgroup can only be spinning while it holds a consumer tile, and the producer tiles
//    it waits for are held by resident workgroups that never wait or are still ahead of every
//    consumer in their queue, so every semaphore is eventually posted whatever the dispatcher
//    does.  (Tiles named by the block index instead, hw_order_tile, are for launches whose
//    tiles are all resident at once, or at the caller's explicit request.)
//  * post: every wave drains its write-through stores, the workgroup meets at a barrier, one
//    lane increments the tile's semaphore at agent scope (Section III-D).
//  * wait: every wave polls the same semaphore word (all lanes read one address, the result
//    is made scalar, so the spin loop is wave-uniform) and sleeps between polls.  No lane-0
//    branch, no extra barrier, and no cache invalidate (see dep_wait in gemm_tile.hpp for why
//    none is needed).
#pragma once
#include <hip/hip_runtime.h>
#include "chain_args.h"
#include "dep_map.hpp"

namespace depsync {

#define DS_FLAG_NO_REORDER 1u
#define DS_FLAG_COUNT 2u
#define DS_FLAG_REVERSE_ORDER 4u
#define DS_FLAG_HW_ORDER 8u
#define DS_FLAG_TRACE 16u

// One look at a semaphore.  The load is a relaxed atomic; the compiler fence behind it keeps
// every later memory operation of the wave (the requests for the tiles being waited for) behind
// the look.  On the hardware side loads return in issue order and the wave acts on the value
// only after it has arrived, caches are invalidated at kernel start, and a line of an
// intermediate is never read before its producer has posted: no cache invalidate is needed.
__device__ __forceinline__ uint32_t sem_load(const uint32_t* sem) {
    uint32_t v = __hip_atomic_load(sem, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __atomic_signal_fence(__ATOMIC_ACQUIRE);
    return __builtin_amdgcn_readfirstlane(v);
}

__device__ __forceinline__ bool sem_reached(uint32_t v, uint32_t target) {
    return (int32_t)(v - target) >= 0;
}

// State one wave keeps while it runs a tile.
struct WaitCtx {
    const ChainArgs* args;
    uint32_t ticket;     // relative ticket of the tile (for the status block)
    bool ok;             // false once a bounded wait expired: the tile's stores are skipped
};

__device__ __forceinline__ uint64_t now_ticks() { return __builtin_amdgcn_s_memrealtime(); }

__device__ __forceinline__ uint32_t hw_where(uint32_t stage) {
    uint32_t xcc, hw;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID, 0, 4)" : "=s"(xcc));
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID, 0, 32)" : "=s"(hw));
    const uint32_t cu = (hw >> 8) & 15u, se = (hw >> 13) & 7u;
    return stage | ((xcc & 15u) << 8) | (cu << 16) | (se << 24);
}

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
    uint32_t nap = 0;
    while (!sem_reached(v, target)) {
        // back off: 2, 4, 8, then 16 units of 64 clocks (about 0.5 us) between polls: a producer
        // tile of a short chain lasts a few microseconds, and a wave that sleeps through its
        // post adds the rest of its nap to the chain; waiting waves poll a few dozen
        // different lines, which the L2 serves without trouble at that rate
        if (nap == 0) __builtin_amdgcn_s_sleep(2);
        else if (nap == 1) __builtin_amdgcn_s_sleep(4);
        else if (nap == 2) __builtin_amdgcn_s_sleep(8);
        else __builtin_amdgcn_s_sleep(16);
        ++nap;
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

// post (Section III-D): called by all threads of the workgroup after the tile's stores.
template <bool THROUGH>
__device__ __forceinline__ void post_tile(const ChainArgs& a, const StageDesc& s, uint32_t tile_lin, uint32_t x, uint32_t y) {
    if (s.post_kind == DEP_NONE) return;
    // every wave's (write-through) stores have completed before the barrier
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        if (a.delay_tile == tile_lin + 1) {
            for (uint32_t i = 0; i < a.delay_iters; ++i) __builtin_amdgcn_s_sleep(127);
        }
        uint32_t idx = policy_sem(s.post_kind, x, y, s.grid_y, s.post_stride);
        // Release: the tile's output was stored with agent-scope (write-through) stores, all of
        // which have completed (vmcnt(0) of every wave, then the barrier), so no write-back of
        // the L2 is needed before the semaphore moves; a relaxed increment is enough.  (A
        // release-ordered atomic would write the whole L2 back, and the compiler drops the wait
        // between that write-back and the increment when it sees no vector memory operation
        // pending, which let consumers on other XCDs read stale memory.)  A tile that was stored
        // with ordinary stores has the write-back and its wait spelled out here.
        if constexpr (!THROUGH) asm volatile("buffer_wbl2 sc1\n\ts_waitcnt vmcnt(0)" ::: "memory");
        __hip_atomic_fetch_add(&s.post_sems[idx * SYNC_WORD_STRIDE], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (a.flags & DS_FLAG_COUNT)
            __hip_atomic_fetch_add(&a.status->posts, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// The tile a workgroup runs.
struct TileId {
    uint32_t stage, tx, ty;   // ty counts rows of the dispatch grid: row tile * ksplit + K part
    uint32_t rel;      // first_ticket[stage] + row-major index: unique per tile, used in the status
};

__device__ __forceinline__ uint32_t xcc_id() {
    uint32_t x;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID, 0, 4)" : "=s"(x));
    return x & 7u;
}

// Tile dispatch (Sections III-B and III-C).  Every stage has one queue per XCD (each XCD has
// its own L2): queue q of a stage holds the stage's tiles whose column tile index is congruent
// to q mod 8, in row-major order, so that the tiles an XCD works on share operand rows and
// columns.  A stage with fewer than 8 column tiles (a convolution with few output channels)
// would leave queues empty that way; there queue q holds the tiles whose row-major index is
// congruent to q mod 8.  A workgroup of ANY launch of the chain takes a tile of the earliest stage that
// still has undrawn tiles, from the queue of the XCD it runs on if that one is not empty, else
// from the next non-empty one.  Hence no consumer tile is handed out while a producer tile is
// undrawn anywhere: a workgroup can only be waiting when every tile of the stage it waits for
// is already held by a resident workgroup, and by induction over the stages those finish.
// A queue counter only grows: entry = counter - queue_epoch * queue_length; a draw beyond the end
// is undone, so after a chain every counter has advanced by exactly its queue length.
__device__ __forceinline__ uint32_t queue_len(const StageDesc& st, uint32_t q) {
    const uint32_t rows = st.grid_y * st.ksplit;
    return st.queue_by_col ? ((st.grid_x + 7u - q) >> 3) * rows : (st.grid_x * rows + 7u - q) >> 3;
}
// Entry i of queue q -> tile (tx, ty).
__device__ __forceinline__ void queue_entry(const StageDesc& st, uint32_t q, uint32_t i, uint32_t& tx, uint32_t& ty) {
    if (st.queue_by_col) {
        const uint32_t ncol = (st.grid_x + 7u - q) >> 3;
        ty = i / ncol; tx = q + 8u * (i % ncol);
    } else {
        const uint32_t lin = q + 8u * i;
        ty = lin / st.grid_x; tx = lin % st.grid_x;
    }
}

// Tile named by the hardware's block index (hooks compiled out, or DEPSYNC_FLAG_HW_ORDER).
__device__ __forceinline__ TileId hw_order_tile(const ChainArgs& a) {
    TileId t;
    const uint32_t rel = a.block_offset + blockIdx.x;
    uint32_t stage = 0;
    if (a.n_stages > 1 && rel >= a.first_ticket[1]) stage = 1;
    if (a.n_stages > 2 && rel >= a.first_ticket[2]) stage = 2;
    if (a.n_stages > 3 && rel >= a.first_ticket[3]) stage = 3;
    const uint32_t lin = rel - a.first_ticket[stage], gx = a.st[stage].grid_x;
    t.stage = stage; t.tx = lin % gx; t.ty = lin / gx; t.rel = rel;
    return t;
}

// Dispatch state of one workgroup.  Workgroups are persistent: a launch has no more of them
// than fit on the chip at once and each keeps drawing tiles until the stages it may work on
// (stage_lo..stage_hi of the launch) are handed out.  That keeps the XCDs balanced whatever
// the tiles' durations are: workgroup i always runs on XCD i mod 8, so with one workgroup per
// tile an XCD that happened to get the long tiles would still have to run its share of the
// rest.  The draws are made by the first lane of wave 1 (wave 0's first lane does the post).
//
// Traffic on the counters' lines is what a draw costs when thousands of workgroups draw (reads
// and increments of one line are served one after the other: 2048 workgroups that each read
// all eight counters per tile made a chain of 64 KiB copy tiles take 213 us instead of 89).
// So in the steady state a draw is ONE increment of the queue the workgroup drew from last,
// started during the current tile's stores (grab) and collected when the tile is done.  The
// counters are only read where a blind increment would probably fail: near the end of the
// queue peek reads that queue's counter when the tile's main loop ends; if it shows the queue
// empty, grab starts reading all eight, so that draw can pick another queue (or move on to
// the next stage) without a round trip for the look; and after a failed increment.  A failed
// increment is undone.
constexpr uint32_t DRAW_THREAD = 64;

struct Drawer {
    const ChainArgs& a;
    uint32_t* slot;        // four words of LDS used to broadcast a tile to the workgroup
    uint32_t home;         // XCD this workgroup runs on
    uint32_t open;         // first stage not yet known to be handed out completely
    uint32_t cur_q;        // queue of stage `open` this workgroup drew from last
    uint32_t last_i;       // entry it got there (0xffffffff: none yet in this stage)
    uint32_t c0;           // counter of (open, cur_q) as read by peek()
    uint32_t c[8];         // counters of stage `open` as read by grab() when c0 showed the queue empty
    bool peeked;           // c0 is being read
    bool looked;           // c[] is being read
    bool first;
    bool pending;          // grab() has an increment in flight
    uint32_t pend_q, pend_val;

    __device__ __forceinline__ Drawer(const ChainArgs& args, uint32_t* lds_slot)
        : a(args), slot(lds_slot), home(xcc_id()), open(args.stage_lo), cur_q(home), last_i(0xffffffffu),
          peeked(false), looked(false), first(true), pending(false), pend_q(0), pend_val(0) {}

    __device__ __forceinline__ uint32_t* counter(uint32_t q) const { return a.ticket + (8u * open + q) * SYNC_WORD_STRIDE; }
    __device__ __forceinline__ uint32_t base(uint32_t len) const { return a.queue_epoch * len; }

    // Is the queue this workgroup draws from close enough to its end that a blind increment
    // would probably fail?  (As many entries left as workgroups may be drawing from it.)
    __device__ __forceinline__ bool near_end() const {
        if (last_i == 0xffffffffu) return false;
        const uint32_t len = queue_len(a.st[open], cur_q);
        return last_i + (gridDim.x >> 3) + 2u >= len;
    }

    // Entries left in the queues of stage `open`, one bit per queue, by the counters in c[].
    __device__ __forceinline__ uint32_t available() const {
        uint32_t avail = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t len = queue_len(a.st[open], j);
            if (c[j] - base(len) < len) avail |= 1u << j;
        }
        return avail;
    }
    __device__ __forceinline__ uint32_t first_from_home(uint32_t avail) const {
        const uint32_t rot = (avail >> home) | (avail << (8u - home));
        return (home + (uint32_t)__builtin_ctz(rot & 0xffu)) & 7u;
    }

    __device__ __forceinline__ void look() {
#pragma unroll
        for (int j = 0; j < 8; ++j) c[j] = __hip_atomic_load(counter(j), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        looked = true;
    }

    // When the tile's main loop ends.  Away from the end of the queue the increment for the next
    // tile starts here already: it is served at the memory side, one workgroup of the XCD after
    // the other, and the tile's stores are followed by a wait for everything the wave has in
    // flight, so an increment started during the stores holds up the post (measured on the GPT-3
    // chain at 2048 tokens: the tiles of a queue-order launch ended 1-2 us later than the same
    // tiles named by the block index).  Near the end of the queue only its counter is read (the
    // value is not looked at here, so the load stays in flight behind what the wave does next).
    __device__ __forceinline__ void peek() {
        if (threadIdx.x != DRAW_THREAD || open > a.stage_hi) return;
        if (!near_end()) { start_increment(); return; }
        c0 = __hip_atomic_load(counter(cur_q), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        peeked = true;
    }

    __device__ __forceinline__ void start_increment() {
        if (pending || a.draw_cas || queue_len(a.st[open], cur_q) == 0) return;
        pend_q = cur_q;
        pend_val = __hip_atomic_fetch_add(counter(cur_q), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        pending = true;
    }

    // A while later (before the tile's stores): near the end of the queue, start the increment for
    // the next tile on the queue drawn from last if the counter read by peek() shows entries,
    // else start reading all eight counters for draw().  (Elsewhere peek() has started it.)
    __device__ __forceinline__ void grab() {
        if (threadIdx.x != DRAW_THREAD || open > a.stage_hi || pending || a.draw_cas) return;
        const uint32_t len = queue_len(a.st[open], cur_q);
        if (near_end()) {
            if (!peeked) return;                              // draw() will look first
            peeked = false;
            if (c0 - base(len) >= len) { look(); return; }    // empty: draw() picks another queue or moves on
        }
        start_increment();
    }

    __device__ __forceinline__ bool take(uint32_t q, uint32_t val, uint32_t& stage, uint32_t& tx, uint32_t& ty) {
        const StageDesc& st = a.st[open];
        const uint32_t len = queue_len(st, q);
        uint32_t i = val - base(len);
        if (i >= len) {                                       // emptied before this increment: undo it
            __hip_atomic_fetch_sub(counter(q), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return false;
        }
        cur_q = q; last_i = i;
        if (open == 0 && (a.flags & DS_FLAG_REVERSE_ORDER)) i = len - 1u - i;
        stage = open; queue_entry(st, q, i, tx, ty);
        return true;
    }

    // DRAW_THREAD, launches that may run late (into a later chain on the same workspace): look at
    // the counters, and take an entry only by compare-and-swap on a value seen to lie inside this
    // chain's part of the counter's range.  Such a launch never moves a counter of another chain.
    __device__ __forceinline__ bool draw_late(uint32_t& stage, uint32_t& tx, uint32_t& ty) {
        for (; open <= a.stage_hi; ++open, cur_q = home) {
            const StageDesc& st = a.st[open];
            bool all = false;                                  // look at the queue drawn from last first, then at all eight
            for (;;) {
                uint32_t q = cur_q, seen;
                if (!all) {
                    seen = __hip_atomic_load(counter(q), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (seen - base(queue_len(st, q)) >= queue_len(st, q)) { all = true; continue; }
                } else {
                    look();
                    const uint32_t avail = available();
                    if (avail == 0) break;                    // handed out (or a later chain's): next stage
                    q = first_from_home(avail);
                    seen = 0;                                  // c[q] without indexing the array by a run-time value
#pragma unroll
                    for (int j = 0; j < 8; ++j) seen = (uint32_t)j == q ? c[j] : seen;
                }
                const uint32_t len = queue_len(st, q);
                uint32_t expected = seen;
                if (__hip_atomic_compare_exchange_strong(counter(q), &expected, seen + 1u, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                         __HIP_MEMORY_SCOPE_AGENT)) {
                    uint32_t i = seen - base(len);
                    cur_q = q; last_i = i;
                    if (open == 0 && (a.flags & DS_FLAG_REVERSE_ORDER)) i = len - 1u - i;
                    stage = open; queue_entry(st, q, i, tx, ty);
                    return true;
                }
            }
        }
        return false;
    }

    // DRAW_THREAD: draw a tile (blocking).
    __device__ __forceinline__ bool draw(uint32_t& stage, uint32_t& tx, uint32_t& ty) {
        if (a.draw_cas) return draw_late(stage, tx, ty);
        // a workgroup launched for the first stage it may work on goes straight for its XCD's
        // queue the first time (one round trip); so does every workgroup that moves on to a
        // stage with at least a tile for each of them
        bool direct = first && a.block_offset + blockIdx.x < a.first_ticket[a.stage_lo + 1];
        first = false;
        peeked = false;
        if (pending) {                                       // the increment grab() started
            pending = false;
            if (take(pend_q, pend_val, stage, tx, ty)) return true;
        }
        bool fresh = false;                                  // moved on to this stage just now
        for (; open <= a.stage_hi; ++open, cur_q = home, last_i = 0xffffffffu, fresh = true) {
            const StageDesc& st = a.st[open];
            // blind only where every workgroup of the launch can get a tile of the stage
            if (fresh) direct = st.grid_x * st.grid_y * st.ksplit >= gridDim.x;
            for (uint32_t attempt = 0; attempt < 16; ++attempt) {
                uint32_t q = home;
                if (!direct || queue_len(st, home) == 0) {
                    if (!looked) look();
                    looked = false;                              // one look serves one attempt
                    const uint32_t avail = available();
                    if (avail == 0) break;                       // stage handed out: next stage
                    q = first_from_home(avail);
                }
                direct = false;
                const uint32_t val = __hip_atomic_fetch_add(counter(q), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (take(q, val, stage, tx, ty)) return true;    // else emptied in the meantime: look again
            }
            // 16 lost races in a row: whatever is left of this stage is being taken by others
        }
        return false;
    }

    // All threads: the next tile of this workgroup (rel = 0xffffffff when there is none).
    __device__ __forceinline__ TileId next() {
        __syncthreads();   // the slot is part of the operand staging area: the last tile is done with it
        if (threadIdx.x == DRAW_THREAD) {
            uint32_t stage = 0, tx = 0, ty = 0;
            const bool found = draw(stage, tx, ty);
            slot[0] = stage; slot[1] = tx; slot[2] = ty; slot[3] = found ? 1u : 0u;
        }
        __syncthreads();
        TileId t;
        t.stage = __builtin_amdgcn_readfirstlane(slot[0]);
        t.tx = __builtin_amdgcn_readfirstlane(slot[1]);
        t.ty = __builtin_amdgcn_readfirstlane(slot[2]);
        const uint32_t found = __builtin_amdgcn_readfirstlane(slot[3]);
        __syncthreads();   // everyone has read the slot before the next tile's operands land on it
        t.rel = found ? a.first_ticket[t.stage] + t.ty * a.st[t.stage].grid_x + t.tx : 0xffffffffu;
        return t;
    }
};

// Stand-in where tiles come from the hardware's block index (nothing to look ahead for).
struct NoDrawer {
    __device__ __forceinline__ void peek() {}
    __device__ __forceinline__ void grab() {}
};

}  // namespace depsync
