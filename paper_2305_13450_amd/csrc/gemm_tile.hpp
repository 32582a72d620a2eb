// One output macro-tile of a GeMM or implicit-GeMM 3x3 convolution on CDNA4 (gfx950):
//   C[m0:m0+TM, n0:n0+TN] = act( A[m0:m0+TM, :] * B[n0:n0+TN, :]^T ),   A, B contiguous along K.
// 256 threads = 4 wave64s in a WM x WN grid; each wave owns a (TM/WM) x (TN/WN) sub-tile built
// from 32x32 accumulator blocks of v_mfma_f32_32x32x16 (bf16 or f16 in, fp32 accumulate).
// Operand tiles of 64 K-elements (128-byte rows) are DMA'd from global memory straight into
// LDS (global_load_lds_dwordx4), two to eight stages deep (a ring per operand), with the 16-byte
// chunks of every row XOR swizzled so that the 128-bit fragment reads are free of bank conflicts.
//
// The tile is the unit the synchronisation subsystem works on (Fig. 4a of the paper): a
// consumer tile waits before loading the slice of A that an earlier stage produces, and a
// producer tile posts after its stores.  The independent operand B (weights) is requested
// before the wait (the load/wait reordering of Section IV-C).
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

#include "chain_args.h"
#include "dep_map.hpp"
#include "sync_device.hpp"

namespace depsync {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int TM_, int TN_, int WM_, int WN_, int MINB_, int NSTAGE_, int NSTB_ = 0>
struct TileCfg {
    static constexpr int TM = TM_, TN = TN_, WM = WM_, WN = WN_, MINB = MINB_;
    static constexpr int BK = 64;                     // K elements per pipeline step
    static constexpr int ROWB = BK * 2;               // bytes per LDS row: one 128-byte line of the operand
    static constexpr int KK = BK / 16;                // 16-wide K slices (one MFMA deep) per step
    static constexpr int RPD = 1024 / ROWB;           // operand rows one 1 KB DMA instruction fills
    static constexpr int LPR = ROWB / 16;             // lanes (16-byte chunks) per row
    static constexpr int NSTAGE = NSTAGE_;               // LDS stages of the A operand: NSTAGE-1 K steps in flight
    static constexpr int NSTB = NSTB_ ? NSTB_ : NSTAGE_; // LDS stages of the B operand (no more than A's)
    static constexpr int WTM = TM / WM, WTN = TN / WN;  // wave sub-tile
    static constexpr int FM = WTM / 32, FN = WTN / 32;  // 32x32 blocks per wave
    static constexpr int NIA = TM / (4 * RPD), NIB = TN / (4 * RPD);  // 1 KB DMA instructions per wave per step
    static constexpr int A_BYTES = TM * ROWB, B_BYTES = TN * ROWB;
    static constexpr int B_BASE = NSTAGE * A_BYTES;      // the B stages follow the A stages
    static constexpr int LDS_BYTES = NSTAGE * A_BYTES + NSTB * B_BYTES;
    static_assert(WM * WN == 4, "four waves per workgroup");
    static_assert(NSTB >= 2 && NSTAGE >= NSTB && MINB * LDS_BYTES <= 160 * 1024, "stages must fit the 160 KB LDS");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile is made of 32x32 blocks");
    static_assert(TM % (4 * RPD) == 0 && TN % (4 * RPD) == 0, "each wave issues whole DMA groups");
};

template <typename T> struct Mma;
template <> struct Mma<__bf16> {
    using V8 = bf16x8;
    static __device__ __forceinline__ f32x16 mma(V8 a, V8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};
template <> struct Mma<_Float16> {
    using V8 = f16x8;
    static __device__ __forceinline__ f32x16 mma(V8 a, V8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
};

// Position swizzle of the 16-byte chunks of LDS row r (128-byte rows).  Any 8 consecutive rows
// get 8 distinct positions (32 banks), and any 16 consecutive rows get 16 distinct (position, row
// parity) pairs (64 banks).  The pattern repeats every 16 rows, so fragment blocks 32 rows apart
// share one per-lane offset.
__device__ __forceinline__ uint32_t swz(uint32_t r) { return (r & 7u) ^ ((r >> 3) & 1u); }

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

__device__ __forceinline__ void dma16(const char* g, char* l) {
    __builtin_amdgcn_global_load_lds((gptr_t)g, (lptr_t)l, 16, 0, 0);
}
// Store one 16-bit output element.  With the synchronisation hooks compiled in, the store is an
// agent-scope store: it is written through this XCD's L2 to memory, so that the post needs no
// write-back of the whole L2 before the semaphore moves.
template <bool THROUGH, typename T>
__device__ __forceinline__ void store_out(T* p, T v) {
    if constexpr (THROUGH) {
        uint16_t bits;
        __builtin_memcpy(&bits, &v, 2);
        __hip_atomic_store(reinterpret_cast<uint16_t*>(p), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        *p = v;
    }
}
// Store eight consecutive 16-bit output elements (16-byte aligned).
template <bool THROUGH, typename V8>
__device__ __forceinline__ void store_out16(void* p, V8 v) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    if constexpr (THROUGH) {
        u32x4 bits;
        __builtin_memcpy(&bits, &v, 16);
        asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(bits) : "memory");
    } else {
        *(V8*)p = v;
    }
}
// GeLU x * Phi(x) with Phi written through erfc: Phi(x) = erfc(-x / sqrt 2) / 2, and for z >= 0
// erfc(z) = t (a1 + t (a2 + t (a3 + t (a4 + t a5)))) exp(-z^2), t = 1 / (1 + p z), to 1.5e-7
// absolute (Abramowitz and Stegun 7.1.26).  Working from erfc on the negative side keeps the
// small values of the left tail free of the cancellation in 1 + erf; the whole thing is two
// transcendental and a dozen plain instructions, less than half of a library erff, which
// matters where the epilogue is not hidden (the workgroup that finishes a tile split along K).
__device__ __forceinline__ float gelu_erf(float x) {
    const float z = fabsf(x) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.3275911f, z, 1.0f));
    float h = __builtin_fmaf(t, 0.5f * 1.061405429f, 0.5f * -1.453152027f);   // coefficients of erfc / 2
    h = __builtin_fmaf(t, h, 0.5f * 1.421413741f);
    h = __builtin_fmaf(t, h, 0.5f * -0.284496736f);
    h = __builtin_fmaf(t, h, 0.5f * 0.254829592f);
    h = h * t * __builtin_amdgcn_exp2f(z * z * -1.4426950408889634f);          // erfc(z) / 2 = Phi(-|x|)
    return x * (x >= 0.0f ? 1.0f - h : h);
}
__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + __expf(-x)); }

// ---- dependency bookkeeping of a consumer tile -------------------------------------------

// Wait for the semaphores of one dependency segment.  Acquire ordering without a cache
// invalidate: the semaphore reads are agent-scope atomic loads whose values this wave branches
// on before it issues the dependent operand's loads.  Those loads cannot hit a stale line in
// this XCD's L2: caches are invalidated when a kernel starts, nothing reads a line of the
// intermediate before the tile that produces it has posted, and the host requires the
// intermediate's rows to be 128-byte aligned, so a cache line never mixes the outputs of two
// producer tiles.
__device__ __forceinline__ void dep_wait(WaitCtx& w, const StageDesc& s, const DepRange& r) {
    const uint32_t target = s.sem_target_base + s.sem_value;
    for (uint32_t y = r.y0; y <= r.y1; ++y) {
        const uint32_t* sem = s.sems + policy_sem(s.dep_kind, r.x, y, s.prod_grid_y, s.stride) * SYNC_WORD_STRIDE;
        const uint32_t v = sem_load(sem);
        if (!sem_reached(v, target)) sem_wait(w, sem, target, v);
    }
}

// ---- the tile ------------------------------------------------------------------------------

// A wave-uniform value pinned into scalar registers (so that the compiler keeps it there
// instead of re-reading kernel arguments inside the K loop).
__device__ __forceinline__ uint32_t uni(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ const char* uni_ptr(const void* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint64_t lo = uni((uint32_t)v), hi = uni((uint32_t)(v >> 32));
    return reinterpret_cast<const char*>(lo | (hi << 32));
}

// DEP != 0: this tile's A operand is produced by the previous stage of the chain (the tile waits
// on semaphores before it requests a slice of A).  DEP == 1: everything it depends on is waited
// for before its first slice (RowSync, and the convolution's whole-halo wait), so the K loop is
// the one of a tile without dependencies; DEP == 2: new dependency segments start inside the K
// loop (TileSync, StridedSync, the convolution's per-filter-row waits).
// THROUGH: the tile's output is waited for by a later stage and is stored write-through.
template <class Cfg, typename T, bool SYNC, uint32_t AMODE, int DEP, bool THROUGH, class DR>
__device__ __forceinline__ void gemm_tile(const ChainArgs& args, const StageDesc& s, uint32_t tx, uint32_t tyz,
                                          uint32_t rel_ticket, char* lds, uint64_t t_enter, DR& dr) {
    using M = Mma<T>;
    using V8 = typename M::V8;
    constexpr int TM = Cfg::TM, TN = Cfg::TN, FM = Cfg::FM, FN = Cfg::FN;
    constexpr int NIA = Cfg::NIA, NIB = Cfg::NIB;
    static_assert(!DEP || SYNC, "dependencies exist only with the synchronisation hooks compiled in");
    // A tile whose output a later stage waits for stores it write-through, so that the post needs
    // no write-back of the L2: a chain's first stage, and the middle stages of a chain of three or
    // four convolutions.  The last stage stores normally.  (A posting tile instantiated without
    // THROUGH still works: post_tile then writes the L2 back for it.)
    static_assert(!THROUGH || SYNC, "write-through stores belong to the synchronised kernels");

    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = uni(tid >> 6);
    const uint32_t wm = wave / Cfg::WN, wn = wave % Cfg::WN;
    const uint32_t sM = uni(s.M), sN = uni(s.N);
    const bool gate_up = (s.bmode == B_GATE_UP);
    const uint32_t tn_out = gate_up ? TN / 2 : TN;       // output columns this tile owns
    const uint32_t S = uni(s.ksplit);                      // workgroups per output tile (split along K)
    const uint32_t ty = tyz / S, kz = tyz % S;
    const uint32_t m0 = ty * TM, n0 = tx * tn_out;
    constexpr uint32_t BK = Cfg::BK, ROWB = Cfg::ROWB;
    const uint32_t KT = uni(s.K / BK);
    const uint32_t kb = kz * (KT / S), ke = kb + KT / S;   // this workgroup's K steps
    const char* const Abase = uni_ptr(s.A);
    const char* const Bbase = uni_ptr(s.B);
    const uint32_t bkstep = uni(s.b_kstep_bytes);
    // conv geometry (unused otherwise)
    const uint32_t cH = uni(s.H), cW = uni(s.W), cCin = uni(s.Cin);
    const char* const zero_page = uni_ptr(s.zero_page);

    WaitCtx wctx{&args, rel_ticket, true};
    const bool tracing = SYNC && (args.flags & DS_FLAG_TRACE) && args.trace != nullptr && rel_ticket < args.trace_cap;
    uint64_t t_start = 0, t_ready = 0;
    if (tracing) t_start = now_ticks();

    // ---- per-lane DMA source offsets (bytes from the operand base, K step 0) ----
    const uint32_t lrow = lane / Cfg::LPR, lpos = lane % Cfg::LPR;
    uint32_t offA[NIA], offB[NIB];
    uint32_t pixyx[AMODE == A_CONV3X3 ? NIA : 1];   // conv: (y << 16) | x of the output pixel of each DMA row
#pragma unroll
    for (int i = 0; i < NIA; ++i) {
        const uint32_t r = (wave * NIA + i) * Cfg::RPD + lrow;
        const uint32_t c = lpos ^ swz(r);
        const uint32_t m = min(m0 + r, sM - 1);
        offA[i] = m * s.lda * 2u + c * 16u;
        if constexpr (AMODE == A_CONV3X3) {
            const uint32_t rem = m % (cH * cW);
            pixyx[i] = ((rem / cW) << 16) | (rem % cW);
        }
    }
#pragma unroll
    for (int i = 0; i < NIB; ++i) {
        const uint32_t q = (wave * NIB + i) * Cfg::RPD + lrow;
        const uint32_t c = lpos ^ swz(q);
        uint32_t row;
        if (gate_up) {
            const uint32_t blk = q >> 5, within = q & 31u;
            const uint32_t col = min(n0 + (blk >> 1) * 32 + within, sN - 1);
            row = (blk & 1u) * sN + col;
        } else {
            row = min(n0 + q, sN - 1);
        }
        offB[i] = row * s.b_row_bytes + c * 16u;
    }

    // Source of the K step that is being requested ("next" step): a byte offset for B and the
    // dense A, and for the conv the filter tap (fr, fs in -1..1) and the byte shift of that tap.
    struct NextStep {
        uint32_t kbytes;     // byte offset of the K step in a row of A
        uint32_t kbytes_b;   // byte offset of the K step in B
        uint32_t tap, c0;    // conv: filter tap 0..8 and first input channel of the step
        int fr, fs;
        long shift;
    } nx;
    // (A and B may be requested a different number of steps ahead, so each has its own "next")
    auto set_next_A = [&](uint32_t kt) __attribute__((always_inline)) {
        nx.kbytes = kt * ROWB;
        if constexpr (AMODE == A_CONV3X3) {
            const uint32_t k0 = kt * BK;
            nx.tap = k0 / cCin; nx.c0 = k0 % cCin;
            nx.fr = (int)(nx.tap / 3) - 1; nx.fs = (int)(nx.tap % 3) - 1;
            nx.shift = ((long)nx.fr * (long)cW + nx.fs) * (long)cCin * 2 + (long)nx.c0 * 2;
        }
    };
    auto set_next_B = [&](uint32_t kt) __attribute__((always_inline)) {
        nx.kbytes_b = kt * bkstep;
    };
    // One 1 KB DMA instruction of the B (weights) or A operand of the next K step into `stage`.
    auto dma_B = [&](uint32_t stage, int i) __attribute__((always_inline)) {
        char* l = lds + Cfg::B_BASE + stage * Cfg::B_BYTES + wave * (NIB * 1024);
        dma16(Bbase + nx.kbytes_b + offB[i], l + i * 1024);
    };
    auto dma_A = [&](uint32_t stage, int i) __attribute__((always_inline)) {
        char* l = lds + stage * Cfg::A_BYTES + wave * (NIA * 1024);
        const char* src;
        if constexpr (AMODE == A_CONV3X3) {
            const int y = (int)(pixyx[i] >> 16) + nx.fr, x = (int)(pixyx[i] & 0xffffu) + nx.fs;
            const bool valid = (y >= 0) && (y < (int)cH) && (x >= 0) && (x < (int)cW);
            src = valid ? Abase + nx.shift + offA[i] : zero_page + lpos * 16u;
        } else {
            src = Abase + nx.kbytes + offA[i];
        }
        dma16(src, l + i * 1024);
    };
    auto issue_B = [&](uint32_t stage) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NIB; ++i) dma_B(stage, i);
    };
    auto issue_A = [&](uint32_t stage) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NIA; ++i) dma_A(stage, i);
    };

    // ---- per-lane fragment read offsets (bytes inside the A / B part of a stage) ----
    constexpr int KK = Cfg::KK;
    uint32_t aoff[KK], boff[KK];
    {
        const uint32_t ra = wm * Cfg::WTM + (lane & 31u), rb = wn * Cfg::WTN + (lane & 31u);
        const uint32_t h = lane >> 5;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            aoff[kk] = ra * ROWB + ((((uint32_t)kk * 2u + h) ^ swz(ra)) << 4);
            boff[kk] = rb * ROWB + ((((uint32_t)kk * 2u + h) ^ swz(rb)) << 4);
        }
    }

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const bool reorder = !(args.flags & DS_FLAG_NO_REORDER);

    // Dependency segments start at multiples of seg_steps K steps (0: only at step 0).
    uint32_t seg_steps = 0, seg_next = kb;   // the host makes K ranges start on segment boundaries
    if constexpr (DEP == 2) seg_steps = uni(dep_seg_steps(s));
    // Called before the A slice of K step k (< KT) is requested into `stage`: if a dependency
    // segment starts there, make sure its producer tiles have posted.  The semaphores are looked
    // at 64 segments at a time (lane l tests the segment l places ahead, one load instruction
    // for the wave), so a tile whose producers are long done pays one round trip for its whole
    // K loop instead of one per segment.  When the segment at hand has not been posted, the
    // weights of the step are requested first (the load/wait reordering) and then the wave
    // really waits; the caller requests the slice (and, harmlessly, the weights again) afterwards.
    uint32_t ready_until = 0;      // every segment that starts before this K step is known to be posted
    auto dep_before_request = [&](uint32_t k, uint32_t stage, bool b_due) __attribute__((always_inline)) {
        if constexpr (DEP) {
            // (rare: the K loop's common path must stay one straight run of code; with the check's
            // branches laid out between the hand-over and the slices, the three taken jumps per step
            // cost the dependent tiles 7 % on a 256x192 tile)
            if (__builtin_expect(k == seg_next, 0)) {
                seg_next = seg_steps ? seg_next + seg_steps : 0xffffffffu;
                DepRange dr;
                if (!dep_segment(s, m0, TM, k, kb, dr)) return;
                bool polled = false;
                if (k >= ready_until) {
                    const uint32_t ka = k + lane * seg_steps;          // lane's segment start
                    bool ok = true;
                    DepRange la;
                    if (ka < ke && (lane == 0 || seg_steps != 0) && dep_segment(s, m0, TM, ka, kb, la)) {
                        const uint32_t target = s.sem_target_base + s.sem_value;
                        for (uint32_t y = la.y0; y <= la.y1; ++y) {
                            const uint32_t* sem = s.sems + policy_sem(s.dep_kind, la.x, y, s.prod_grid_y, s.stride) * SYNC_WORD_STRIDE;
                            ok = ok && sem_reached(__hip_atomic_load(sem, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT), target);
                        }
                    }
                    const uint64_t mask = __ballot(ok);
                    // the requests for the dependent slice stay behind the look at its semaphores:
                    // a compiler fence (the loads are relaxed atomics, which the compiler may
                    // otherwise reorder with ordinary memory operations); the hardware returns
                    // loads in issue order, and the wave acts on the values only after they arrived
                    __atomic_signal_fence(__ATOMIC_ACQUIRE);
                    const uint32_t n_ready = (~mask == 0) ? 64u : (uint32_t)__builtin_ctzll(~mask);
                    if (n_ready == 0) {
                        if (reorder && b_due) issue_B(stage);
                        dep_wait(wctx, s, dr);
                        polled = true;
                        ready_until = k + 1;
                    } else {
                        ready_until = seg_steps ? k + n_ready * seg_steps : 0xffffffffu;
                        // the segments seen posted need no further look: the next check is due where
                        // they end (unless every wait is being counted)
                        if (!(args.flags & DS_FLAG_COUNT)) seg_next = ready_until;
                    }
                }
                if (args.flags & DS_FLAG_COUNT) {
                    for (uint32_t y = dr.y0; y <= dr.y1; ++y) count_wait(args, polled);
                }
            }
        }
    };

    // ---- prologue ----
    // A is requested NSA-1 steps ahead into a ring of NSA stages, B NSB-1 steps ahead into a ring
    // of NSB <= NSA stages (a tile too large for three stages of both keeps three of A and two of B:
    // then only B's requests of a step, issued first, have to land within the step, and A's
    // are spread over the rest of it with a step more to land).
    constexpr int NSA = Cfg::NSTAGE, NSB = Cfg::NSTB;
    constexpr int NG = KK * FM;           // MFMA groups per step
    constexpr int ND = NIA + NIB;         // DMA instructions per step
    // groups the DMA instructions are spread over: with two stages the step's requests must
    // have landed by the end of the same step, so they go out at its start (measured on the
    // GPT-3 chain at M = 2048: 128x192 601 -> 581 us, 128x128 727 -> 669 us with all of them in
    // the first group; the 256-row tiles, with twice the requests per wave, do best with a
    // quarter of the groups: 256x192 714 -> 684 us)
    constexpr int NGD = (NSA > 2) ? NG : (FM <= 2 ? 1 : NG / 4);
    // Tiles that have a CU to themselves (one wave per SIMD) read all fragments of the next
    // 16-wide K slice together, a whole slice of MFMAs before their first use, with the order
    // pinned: left to itself the compiler issues each read right before the wait for it (while
    // LDS DMA is in flight it only ever waits for lgkmcnt(0)), and with no second workgroup on
    // the CU nothing fills that round trip.  Measured on the GPT-3 chain at M = 2048: 256x128
    // 609 -> 585 us, 256x192 621 -> 612 us; with two workgroups per CU it gains nothing.
    constexpr bool S2 = (Cfg::MINB == 1);
    // At the top of step k the requests of A(k) and B(k) must have landed.  Requests complete in
    // issue order, and a step issues B's before A's, so what may still be outstanding is what was
    // issued after B(k): the A requests of that same step when A runs further ahead than B, and
    // the NSB-2 whole steps after it.
    constexpr int OUTSTANDING = (NSA > NSB ? NIA : 0) + (NSB - 2) * ND;
    static_assert(OUTSTANDING <= 48, "outstanding DMA instructions must fit the vmcnt counter");
    // the steps before the loop, in the order the loop itself would have issued them
#pragma unroll
    for (int p = 0; p < NSA - 1; ++p) {
        const int pb = p - (NSA - NSB);    // B's step issued alongside A's step p
        set_next_A(min(kb + (uint32_t)p, ke - 1));
        if (pb >= 0) set_next_B(min(kb + (uint32_t)pb, ke - 1));
        // the weights of the step go out before the look at the semaphores (the load/wait reordering
        // of Section IV-C), so the poll's round trip is not added to their latency
        if (reorder && pb >= 0) issue_B(pb);
        if (kb + (uint32_t)p < ke) dep_before_request(kb + p, pb >= 0 ? pb : 0, false);
        if (p == 0 && tracing) t_ready = now_ticks();
        if (!reorder && pb >= 0) issue_B(pb);
        issue_A(p);
    }

    // The K loop, as one stream of 16-wide K slices (KK per step, each KK*... FM groups of FN MFMAs
    // per wave).  While a slice's MFMAs run, the fragments of the next slice are read from LDS
    // into the other fragment buffer.  The workgroup barrier that hands over a step's stage sits
    // before the LAST slice of the step before it: at that point every wave has read (not yet
    // multiplied) its last fragments of the current stage, so the stage is free for new requests,
    // and the next step's first fragments travel from LDS while the last slice's MFMAs run; no
    // fragment read is exposed at a step boundary.  The DMA instructions a barrier releases (the
    // steps NSB-1 / NSA-1 ahead, weights first) are spread over the first NGD of the NG groups
    // that follow it.  Past the end of K the last step is simply requested again into an idle
    // stage, so the body is free of branches.
    V8 af[2][FM], bf[2][FN];
    auto load_frags = [&](int buf, const char* la, const char* lb, int kk) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < FM; ++i) af[buf][i] = *(const V8*)(la + aoff[kk] + i * (32 * ROWB));
#pragma unroll
        for (int j = 0; j < FN; ++j) bf[buf][j] = *(const V8*)(lb + boff[kk] + j * (32 * ROWB));
    };
    uint32_t reqA = NSA - 1, reqB = NSB - 1;                 // stages the next requests go into
    // DMA instructions of group g (counted from the barrier that released them)
    auto dma_group = [&](int g) __attribute__((always_inline)) {
        if (g < NGD) {
#pragma unroll
            for (int d = (g * ND) / NGD; d < ((g + 1) * ND) / NGD; ++d) {
                if (d < NIB) dma_B(reqB, d);
                else dma_A(reqA, d - NIB);
            }
        }
    };
    // One slice: MFMAs on fragment buffer `buf`; meanwhile read the fragments of slice nkk of the
    // stage at (nla, nlb) into the other buffer (nkk < 0: none) and issue the DMA groups g0 .. g0+FM-1
    // (g0 < 0: none).
    auto slice = [&](int buf, const char* nla, const char* nlb, int nkk, int g0) __attribute__((always_inline)) {
        const int n = buf ^ 1;
        if constexpr (S2) {
            // One wave per SIMD: nothing else fills the matrix unit while this wave issues other
            // instructions, and a run of fragment reads takes longer to issue than one MFMA to
            // execute.  So the order is pinned: after each MFMA at most one fragment read of the
            // next slice (the fragments the next slice needs first go first), DMA instructions at
            // the start of a group.  The empty asm that reads the current slice's fragments is where
            // the compiler's wait for them lands, before anything of this slice is issued.
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
            for (int i = 0; i < FM; ++i) asm volatile("" ::"v"(__builtin_bit_cast(u32x4, af[buf][i])));
#pragma unroll
            for (int j = 0; j < FN; ++j) asm volatile("" ::"v"(__builtin_bit_cast(u32x4, bf[buf][j])));
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                if (g0 >= 0) dma_group(g0 + i);
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    acc[i][j] = M::mma(af[buf][i], bf[buf][j], acc[i][j]);
                    // fragment read number m of the next slice (A0, B0 .. B(FN-1), A1 ..) follows MFMA
                    // number m; a wave tile of fewer MFMAs than fragments reads the rest after the last
                    constexpr int NF = FM + FN, NM = FM * FN;
                    const int m0 = i * FN + j, m1 = (m0 == NM - 1 && NM < NF) ? NF : m0 + 1;
                    if (nkk >= 0) {
#pragma unroll
                        for (int m = m0; m < m1; ++m) {
                            if (m == 0) af[n][0] = *(const V8*)(nla + aoff[nkk]);
                            else if (m <= FN) bf[n][m - 1] = *(const V8*)(nlb + boff[nkk] + (m - 1) * (32 * ROWB));
                            else if (m < NF) af[n][m - FN] = *(const V8*)(nla + aoff[nkk] + (m - FN) * (32 * ROWB));
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            if (nkk >= 0) {
                af[n][i] = *(const V8*)(nla + aoff[nkk] + i * (32 * ROWB));
#pragma unroll
                for (int j = (i * FN) / FM; j < ((i + 1) * FN) / FM; ++j)
                    bf[n][j] = *(const V8*)(nlb + boff[nkk] + j * (32 * ROWB));
            }
            if (g0 >= 0) dma_group(g0 + i);
#pragma unroll
            for (int j = 0; j < FN; ++j) acc[i][j] = M::mma(af[buf][i], bf[buf][j], acc[i][j]);
        }
    };
    // Hand-over of step k's stage: its requests have landed for every wave (requests complete in
    // issue order; a bare s_barrier, since __syncthreads() would also wait for the younger ones),
    // and every wave has finished reading the stage of step k-1.  Then point the requests at the
    // steps ahead of k (after waiting for what the A slice depends on, if a dependency segment starts).
    auto hand_over = [&](uint32_t k) __attribute__((always_inline)) {
        // The sources of the requests this hand-over releases and the test for a dependency
        // segment are scalar arithmetic: done BEFORE the wait and the barrier, where the wave
        // would idle anyway, and passed through the asm statement as operands so that the
        // compiler cannot sink them into the gap between the barrier and the first MFMA behind
        // it (with a branch in that gap it did: the dependent tiles' steps were 7 % slower than
        // the same steps of a tile without dependencies).
        const uint32_t kreq = k + (NSA - 1);
        set_next_A(min(kreq, ke - 1));
        set_next_B(min(k + (NSB - 1), ke - 1));
        uint32_t seg = 0;
        if constexpr (DEP == 2) seg = uni((kreq < ke && kreq == seg_next) ? 1u : 0u);
        nx.kbytes_b = uni(nx.kbytes_b);
        if constexpr (AMODE == A_CONV3X3) {
            uint32_t lo = uni((uint32_t)(uint64_t)nx.shift), hi = uni((uint32_t)((uint64_t)nx.shift >> 32));
            uint32_t fr = uni((uint32_t)nx.fr), fs = uni((uint32_t)nx.fs);
            asm volatile("s_waitcnt vmcnt(%6) lgkmcnt(0)\n\ts_barrier"
                         : "+s"(lo), "+s"(hi), "+s"(fr), "+s"(fs), "+s"(nx.kbytes_b), "+s"(seg) : "n"(OUTSTANDING) : "memory");
            nx.shift = (long)((uint64_t)lo | ((uint64_t)hi << 32));
            nx.fr = (int)fr; nx.fs = (int)fs;
        } else {
            nx.kbytes = uni(nx.kbytes);
            asm volatile("s_waitcnt vmcnt(%3) lgkmcnt(0)\n\ts_barrier"
                         : "+s"(nx.kbytes), "+s"(nx.kbytes_b), "+s"(seg) : "n"(OUTSTANDING) : "memory");
        }
        if constexpr (DEP == 2) {
            if (__builtin_expect(seg != 0, 0)) dep_before_request(kreq, reqB, true);
        }
    };
    auto advance = [&](uint32_t& st, uint32_t n) __attribute__((always_inline)) { st = (st + 1 == n) ? 0 : st + 1; };
    static_assert(KK % 2 == 0, "fragment buffers alternate with the slices");

    // head: step kb's stage is handed over, its requests go out with slices 0 .. KK-2 (the groups
    // that the missing slice before them would have carried are issued at once)
    uint32_t curA = 0, curB = 0;
    hand_over(kb);
    const char* la = lds;
    const char* lb = lds + Cfg::B_BASE;
    load_frags(0, la, lb, 0);
#pragma unroll
    for (int g = 0; g < FM; ++g) dma_group(g);
#pragma unroll
    for (int kk = 0; kk < KK - 1; ++kk) slice(kk & 1, la, lb, kk + 1, (kk + 1) * FM);
    advance(reqA, NSA); advance(reqB, NSB);
    for (uint32_t kt = kb + 1; kt < ke; ++kt) {
        // the last fragments of step kt-1 are in registers: hand over step kt's stage, multiply
        // them while step kt's first fragments are read, then step kt's slices 0 .. KK-2
        hand_over(kt);
        advance(curA, NSA); advance(curB, NSB);
        la = lds + curA * Cfg::A_BYTES;
        lb = lds + Cfg::B_BASE + curB * Cfg::B_BYTES;
        slice((KK - 1) & 1, la, lb, 0, 0);
#pragma unroll
        for (int kk = 0; kk < KK - 1; ++kk) slice(kk & 1, la, lb, kk + 1, (kk + 1) * FM);
        advance(reqA, NSA); advance(reqB, NSB);
    }
    slice((KK - 1) & 1, nullptr, nullptr, -1, -1);   // tail: the last slice of the last step
    // every DMA into LDS has landed before the staging area is given up
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    dr.peek();   // the look at the dispatch queues for this workgroup's next tile travels during the epilogue

    // ---- split-K: leave the partial tile, and carry on only as the last part to arrive ----
    bool finish = true;
    if (S > 1) {
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        const uint32_t tile_lin = ty * s.grid_x + tx;
        float* const part = s.partials + (size_t)tile_lin * S * (TM * TN);
        // fragment order: each lane stores 16 bytes next to its neighbours' (1 KB per instruction),
        // written through to memory so that the count below can follow without a write-back
        // of this XCD's whole L2
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4 v4 = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                    float* dst = part + (size_t)kz * (TM * TN) + ((((i * FN + j) * 4 + q) * 256 + tid) << 2);
                    // (the wait states a store of more than 8 bytes needs after a vector instruction has
                    // written its data registers are not inserted for an asm statement: spelled out)
                    asm volatile("s_nop 1\n\tglobal_store_dwordx4 %0, %1, off sc1" ::"v"(dst), "v"(v4) : "memory");
                }
        // the partial is in memory before the count moves (every wave's stores, then the barrier)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        uint32_t* slot = reinterpret_cast<uint32_t*>(lds);
        if (tid == 0) {
            const uint32_t old = __hip_atomic_fetch_add(s.arrive + tile_lin * SYNC_WORD_STRIDE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            slot[0] = old;
        }
        __syncthreads();
        finish = __builtin_amdgcn_readfirstlane(slot[0]) == S - 1;
        __syncthreads();
        if (finish) {
            // Every part's partial is in memory (each counted after its stores had completed) and none of
            // these lines has been read on this XCD since the kernel started.  Sum in K order,
            // whoever came last, so that the result does not depend on the arrival order.
            if (tid == 0) __hip_atomic_store(s.arrive + tile_lin * SYNC_WORD_STRIDE, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            // The sum is p0 + p1 + p2 + ... from the left.  A finisher that holds part 0 or
            // part 1 starts from its registers (p1 + p0 and p0 + p1 are the same number) and
            // skips reading its own partial back; any other starts from zero and reads them all.
            const bool own = kz <= 1;
            if (!own) {
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
            }
            // The partials were written on other XCDs and come from memory: a read costs a round
            // trip of a couple of microseconds whatever its size, and a skinny chain's tile has
            // little else left to do.  So the loads of as many whole parts as the registers
            // beside the accumulators hold (PARTS_IN_FLIGHT) are issued before the first of them
            // is added; the adds stay in K order.
            constexpr int ACCF = FM * FN * 16;                                   // accumulator floats per lane
            constexpr int ROOM = Cfg::MINB == 1 ? (472 - ACCF < 192 ? 472 - ACCF : 192) : 216 - ACCF;
            constexpr int PARTS_IN_FLIGHT = ROOM / ACCF > 8 ? 8 : ROOM / ACCF;
            if constexpr (PARTS_IN_FLIGHT >= 1) {
                constexpr int NV = FM * FN * 4;                                  // 16-byte loads per lane and part
                for (uint32_t z0 = 0; z0 < S; z0 += PARTS_IN_FLIGHT) {
                    f32x4 t4[PARTS_IN_FLIGHT][NV];
                    // (parts past the end read the last part again and are not added: the loads stay
                    // unconditional, so that all of a batch are in flight together)
#pragma unroll
                    for (int d = 0; d < PARTS_IN_FLIGHT; ++d) {
                        const uint32_t z = min(z0 + d, S - 1);
                        const float* src = part + (size_t)z * (TM * TN) + (tid << 2);
#pragma unroll
                        for (int u = 0; u < NV; ++u) t4[d][u] = *(const f32x4*)(src + ((u * 256) << 2));
                    }
#pragma unroll
                    for (int d = 0; d < PARTS_IN_FLIGHT; ++d) {
                        const uint32_t z = z0 + d;
                        if (z < S && !(own && z == kz)) {
#pragma unroll
                            for (int i = 0; i < FM; ++i)
#pragma unroll
                                for (int j = 0; j < FN; ++j)
#pragma unroll
                                    for (int q = 0; q < 4; ++q)
#pragma unroll
                                        for (int e = 0; e < 4; ++e) acc[i][j][4 * q + e] += t4[d][(i * FN + j) * 4 + q][e];
                        }
                    }
                }
            } else {
                // no room for a whole part: one row of blocks of one part at a time
                for (uint32_t z = 0; z < S; ++z) {
                    if (own && z == kz) continue;
                    const float* src = part + (size_t)z * (TM * TN) + (tid << 2);
#pragma unroll
                    for (int i = 0; i < FM; ++i) {
                        f32x4 t4[FN][4];
#pragma unroll
                        for (int j = 0; j < FN; ++j)
#pragma unroll
                            for (int q = 0; q < 4; ++q) t4[j][q] = *(const f32x4*)(src + ((((i * FN + j) * 4 + q) * 256) << 2));
#pragma unroll
                        for (int j = 0; j < FN; ++j)
#pragma unroll
                            for (int q = 0; q < 4; ++q)
#pragma unroll
                                for (int e = 0; e < 4; ++e) acc[i][j][4 * q + e] += t4[j][q][e];
                    }
                }
            }
        }
    }

    // ---- epilogue: activation, round to 16 bits, store ----
    // Accumulator layout of the 32x32 block: lane holds column (lane % 32) and rows
    // 8*(v/4) + 4*(lane/32) + v%4 for v = 0..15, i.e. a lane's values run DOWN a column.  Each
    // wave therefore transposes its sub-tile through its own piece of the (now idle) operand
    // staging area and writes it out as 16-byte row segments: a twelfth of the store
    // instructions, and whole lines instead of 2-byte pieces for the write-through stores.
    __syncthreads();   // every wave has read its last operand fragments
    if (wctx.ok && finish) {
        constexpr int PAD = (4 * Cfg::WTM * (Cfg::WTN * 2 + 16) <= Cfg::LDS_BYTES) ? 16 : 0;
        constexpr int PITCH = Cfg::WTN * 2 + PAD;                   // bytes per sub-tile row in LDS
        static_assert(4 * Cfg::WTM * PITCH <= Cfg::LDS_BYTES, "the transposed sub-tiles fit the staging area");
        char* const reg = lds + wave * (Cfg::WTM * PITCH);
        const uint32_t act = s.act;
        const uint32_t colw = lane & 31u, rowh = (lane >> 5) * 4u;
        const uint32_t wtn_out = gate_up ? Cfg::WTN / 2 : Cfg::WTN;  // output columns of this wave
        if (gate_up) {
            if constexpr (FN >= 2) {
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int jp = 0; jp < FN / 2; ++jp)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const uint32_t r = i * 32 + 8 * (v / 4) + rowh + (v % 4), c = jp * 32 + colw;
                            const float g = acc[i][2 * jp][v], u = acc[i][2 * jp + 1][v];
                            *(T*)(reg + r * PITCH + c * 2) = (T)(silu_f(g) * u);
                        }
            }
        } else {
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const uint32_t r = i * 32 + 8 * (v / 4) + rowh + (v % 4), c = j * 32 + colw;
                        float x = acc[i][j][v];
                        if (act == ACT_GELU) x = gelu_erf(x);
                        else if (act == ACT_RELU) x = fmaxf(x, 0.0f);
                        *(T*)(reg + r * PITCH + c * 2) = (T)x;
                    }
        }
        dr.grab();   // the counters read by peek() have arrived by now: start the next tile's draw
        // the region is private to the wave: its own LDS writes are ordered before its reads
        T* Cp = (T*)s.C;
        const uint32_t ldc = s.ldc;
        const uint32_t cpr = wtn_out / 8;                            // 16-byte chunks per row
        const uint32_t row0 = m0 + wm * Cfg::WTM, col0 = n0 + wn * wtn_out;
        for (uint32_t idx = lane; idx < Cfg::WTM * cpr; idx += 64) {
            const uint32_t r = idx / cpr, ch = idx % cpr;
            const uint32_t row = row0 + r, col = col0 + ch * 8;
            if (row >= sM || col >= sN) continue;
            const V8 val = *(const V8*)(reg + r * PITCH + ch * 16);
            T* dst = Cp + (size_t)row * ldc + col;
            if (col + 8 <= sN) {
                store_out16<THROUGH>(dst, val);
            } else {
                for (uint32_t e = 0; e < sN - col; ++e) store_out<THROUGH>(dst + e, (T)val[e]);
            }
        }
    }

    if (SYNC && finish) post_tile<THROUGH>(args, s, ty * s.grid_x + tx, tx, ty);
    if (tracing && tid == 0) {
        TraceRec r;
        r.rel = rel_ticket; r.where = hw_where(DEP ? 1u : 0u); r.tx = tx; r.ty = tyz;
        r.t_enter = t_enter; r.t_start = t_start; r.t_ready = t_ready; r.t_end = now_ticks();
        args.trace[rel_ticket] = r;
    }
}

}  // namespace depsync
