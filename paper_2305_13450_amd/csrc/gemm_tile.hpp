// One output macro-tile of a GeMM or implicit-GeMM 3x3 convolution on CDNA4 (gfx950):
//   C[m0:m0+TM, n0:n0+TN] = act( A[m0:m0+TM, :] * B[n0:n0+TN, :]^T ),   A, B contiguous along K.
// 256 threads = 4 wave64s in a WM x WN grid; each wave owns a (TM/WM) x (TN/WN) sub-tile built
// from 32x32 accumulator blocks of v_mfma_f32_32x32x16 (bf16 or f16 in, fp32 accumulate).
// Operand tiles of 64 K-elements (128-byte rows) are DMA'd from global memory straight into
// LDS (global_load_lds_dwordx4), double-buffered, with the 16-byte chunks of every row XOR
// swizzled so that the 128-bit fragment reads are free of bank conflicts.
//
// The tile is the unit the synchronisation subsystem works on (Fig. 4a of the paper): a
// consumer tile waits before loading the slice of A that an earlier stage produces, and a
// producer tile posts after its stores.  The independent operand B (weights) is requested
// before the wait (the load/wait reordering of Section IV-C).
#pragma once
#include <hip/hip_runtime.h>
#include "chain_args.h"
#include "sync_device.hpp"

namespace depsync {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int TM_, int TN_, int WM_, int WN_, int MINB_>
struct TileCfg {
    static constexpr int TM = TM_, TN = TN_, WM = WM_, WN = WN_, MINB = MINB_;
    static constexpr int BK = 64;                     // K elements per pipeline step
    static constexpr int ROWB = BK * 2;               // bytes per LDS row
    static constexpr int NSTAGE = 2;
    static constexpr int WTM = TM / WM, WTN = TN / WN;  // wave sub-tile
    static constexpr int FM = WTM / 32, FN = WTN / 32;  // 32x32 blocks per wave
    static constexpr int NIA = TM / 32, NIB = TN / 32;  // 1 KB DMA instructions per wave per step
    static constexpr int A_BYTES = TM * ROWB, B_BYTES = TN * ROWB;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
    static_assert(WM * WN == 4, "four waves per workgroup");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile is made of 32x32 blocks");
    static_assert(TM % 32 == 0 && TN % 32 == 0, "each wave issues whole 8-row DMA groups");
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

// Position swizzle of the 16-byte chunks of LDS row r.  Any 8 consecutive rows get 8 distinct
// positions (32 banks), and any 16 consecutive rows get 16 distinct (position, row parity)
// pairs (64 banks).  The pattern repeats every 16 rows, so fragment blocks 32 rows apart share
// one per-lane offset.
__device__ __forceinline__ uint32_t swz(uint32_t r) { return (r & 7u) ^ ((r >> 3) & 1u); }

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

__device__ __forceinline__ void dma16(const char* g, char* l) {
    __builtin_amdgcn_global_load_lds((gptr_t)g, (lptr_t)l, 16, 0, 0);
}

__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }
__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + __expf(-x)); }

// ---- dependency bookkeeping of a consumer tile -------------------------------------------

// Range of producer row tiles and the producer column tile a K step depends on.
struct DepRange {
    uint32_t y0, y1;   // inclusive producer row-tile range
    uint32_t x;        // producer column tile (TILE / STRIDED kinds)
};

// Does the A slice of K step kt start a new dependency segment, and on what?
__device__ __forceinline__ bool dep_segment(const StageDesc& s, uint32_t m0, uint32_t tm, uint32_t kt, DepRange& r) {
    const uint32_t m_last = min(m0 + tm, s.M) - 1;
    switch (s.dep_kind) {
        case DEP_ROW:
            if (kt != 0) return false;
            r.y0 = m0 / s.prod_tm; r.y1 = m_last / s.prod_tm; r.x = 0;
            return true;
        case DEP_TILE:
        case DEP_STRIDED: {
            const uint32_t k0 = kt * 64;
            if (k0 % s.prod_tn != 0) return false;
            r.x = k0 / s.prod_tn;
            if (s.dep_kind == DEP_STRIDED && r.x >= s.stride) return false;  // same semaphore as x - stride
            r.y0 = m0 / s.prod_tm; r.y1 = m_last / s.prod_tm;
            return true;
        }
        case DEP_CONV_ROW: {
            if (kt != 0) return false;
            const int lo = (int)m0 - (int)s.W - 1, hi = (int)m_last + (int)s.W + 1;
            r.y0 = (uint32_t)max(lo, 0) / s.prod_tm;
            r.y1 = (uint32_t)min(hi, (int)s.M - 1) / s.prod_tm; r.x = 0;
            return true;
        }
        case DEP_CONV_TAPROW:
        case DEP_CONV_TILE: {
            // K runs filter-row major: k = ((fr*3 + fs) * Cin + c).  A new segment starts with
            // every filter row (TAPROW) or every producer channel tile of a filter row's first tap (TILE).
            const uint32_t k0 = kt * 64;
            const uint32_t tap = k0 / s.Cin, c0 = k0 % s.Cin;
            const uint32_t fr = tap / 3, fs = tap % 3;
            if (fs != 0) return false;
            if (s.dep_kind == DEP_CONV_TAPROW) { if (c0 != 0) return false; r.x = 0; }
            else { if (c0 % s.prod_tn != 0) return false; r.x = c0 / s.prod_tn; }
            const int sh = ((int)fr - 1) * (int)s.W;
            const int lo = (int)m0 + sh - 1, hi = (int)m_last + sh + 1;
            if (hi < 0 || lo > (int)s.M - 1) return false;      // whole filter row is padding
            r.y0 = (uint32_t)max(lo, 0) / s.prod_tm;
            r.y1 = (uint32_t)min(hi, (int)s.M - 1) / s.prod_tm;
            return true;
        }
        default:
            return false;
    }
}

// Wait (blocking) or test (non-blocking) the semaphores of one dependency segment.  Returns
// true when all are reached; the acquire fence has then been executed.
__device__ __forceinline__ bool dep_wait(WaitCtx& w, const StageDesc& s, const DepRange& r, bool blocking) {
    const uint32_t target = s.sem_target_base + s.sem_value;
    bool polled = false;
    for (uint32_t y = r.y0; y <= r.y1; ++y) {
        const uint32_t* sem = s.sems + policy_sem(s.dep_kind, r.x, y, s.prod_grid_y, s.stride);
        uint32_t v = sem_load(sem);
        if (!sem_reached(v, target)) {
            if (!blocking) return false;
            polled = true;
            sem_wait(w, sem, target, v);
        }
    }
    acquire_agent();
    if (w.args->flags & DS_FLAG_COUNT) {
        for (uint32_t y = r.y0; y <= r.y1; ++y) count_wait(*w.args, polled);
    }
    return true;
}

// ---- the tile ------------------------------------------------------------------------------

template <class Cfg, typename T, bool SYNC, uint32_t AMODE>
__device__ __forceinline__ void gemm_tile(const ChainArgs& args, const StageDesc& s, uint32_t tile_lin,
                                          uint32_t rel_ticket, char* lds) {
    using M = Mma<T>;
    using V8 = typename M::V8;
    constexpr int TM = Cfg::TM, TN = Cfg::TN, FM = Cfg::FM, FN = Cfg::FN;
    constexpr int NIA = Cfg::NIA, NIB = Cfg::NIB;

    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t wm = wave / Cfg::WN, wn = wave % Cfg::WN;
    const uint32_t tx = tile_lin % s.grid_x, ty = tile_lin / s.grid_x;   // row-major, x fastest
    const bool gate_up = (s.bmode == B_GATE_UP);
    const uint32_t tn_out = gate_up ? TN / 2 : TN;       // output columns this tile owns
    const uint32_t m0 = ty * TM, n0 = tx * tn_out;
    const uint32_t KT = s.K / 64;

    WaitCtx wctx{&args, rel_ticket, true};

    // ---- per-lane DMA source offsets (bytes from the operand base, K step 0) ----
    const uint32_t lrow = lane >> 3, lpos = lane & 7u;
    uint32_t offA[NIA], offB[NIB];
    uint32_t pixyx[AMODE == A_CONV3X3 ? NIA : 1];   // conv: (y << 16) | x of the output pixel of each DMA row
#pragma unroll
    for (int i = 0; i < NIA; ++i) {
        const uint32_t r = (wave * NIA + i) * 8 + lrow;
        const uint32_t c = lpos ^ swz(r);
        const uint32_t m = min(m0 + r, s.M - 1);
        offA[i] = m * s.lda * 2u + c * 16u;
        if constexpr (AMODE == A_CONV3X3) {
            const uint32_t rem = m % (s.H * s.W);
            pixyx[i] = ((rem / s.W) << 16) | (rem % s.W);
        }
    }
#pragma unroll
    for (int i = 0; i < NIB; ++i) {
        const uint32_t q = (wave * NIB + i) * 8 + lrow;
        const uint32_t c = lpos ^ swz(q);
        uint32_t row;
        if (gate_up) {
            const uint32_t blk = q >> 5, within = q & 31u;
            const uint32_t col = min(n0 + (blk >> 1) * 32 + within, s.N - 1);
            row = (blk & 1u) * s.N + col;
        } else {
            row = min(n0 + q, s.N - 1);
        }
        offB[i] = row * s.ldb * 2u + c * 16u;
    }

    auto issue_B = [&](uint32_t stage, uint32_t kt) {
        const char* base = (const char*)s.B + (size_t)kt * 128u;
        char* l = lds + stage * Cfg::STAGE_BYTES + Cfg::A_BYTES + wave * (NIB * 1024);
#pragma unroll
        for (int i = 0; i < NIB; ++i) dma16(base + offB[i], l + i * 1024);
    };
    auto issue_A = [&](uint32_t stage, uint32_t kt) {
        char* l = lds + stage * Cfg::STAGE_BYTES + wave * (NIA * 1024);
        if constexpr (AMODE == A_CONV3X3) {
            const uint32_t k0 = kt * 64u;
            const uint32_t tap = k0 / s.Cin, c0 = k0 % s.Cin;
            const int fr = (int)(tap / 3) - 1, fs = (int)(tap % 3) - 1;
            const long shift = ((long)fr * (long)s.W + fs) * (long)s.Cin * 2 + (long)c0 * 2;
            const char* base = (const char*)s.A + shift;
            const char* zero = (const char*)s.zero_page + lpos * 16u;
#pragma unroll
            for (int i = 0; i < NIA; ++i) {
                const int y = (int)(pixyx[i] >> 16) + fr, x = (int)(pixyx[i] & 0xffffu) + fs;
                const bool valid = (y >= 0) && (y < (int)s.H) && (x >= 0) && (x < (int)s.W);
                dma16(valid ? base + offA[i] : zero, l + i * 1024);
            }
        } else {
            const char* base = (const char*)s.A + (size_t)kt * 128u;
#pragma unroll
            for (int i = 0; i < NIA; ++i) dma16(base + offA[i], l + i * 1024);
        }
    };

    // ---- per-lane fragment read offsets (bytes inside the A / B part of a stage) ----
    uint32_t aoff[4], boff[4];
    {
        const uint32_t ra = wm * Cfg::WTM + (lane & 31u), rb = wn * Cfg::WTN + (lane & 31u);
        const uint32_t h = lane >> 5;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            aoff[kk] = ra * 128u + ((((uint32_t)kk * 2u + h) ^ swz(ra)) << 4);
            boff[kk] = rb * 128u + ((((uint32_t)kk * 2u + h) ^ swz(rb)) << 4);
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
    const bool has_dep = SYNC && (s.dep_kind != DEP_NONE);

    // ---- prologue: K step 0 into stage 0 ----
    {
        DepRange dr;
        const bool need = has_dep && dep_segment(s, m0, TM, 0, dr);
        if (need && !reorder) dep_wait(wctx, s, dr, true);
        issue_B(0, 0);
        if (need && reorder) dep_wait(wctx, s, dr, true);
        issue_A(0, 0);
    }

    for (uint32_t kt = 0; kt < KT; ++kt) {
        const uint32_t cur = kt & 1u;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();   // stage `cur` is complete; nobody still reads stage cur^1

        bool pend_a = false, pend_b = false;
        DepRange dr;
        if (kt + 1 < KT) {
            const bool need = has_dep && dep_segment(s, m0, TM, kt + 1, dr);
            const bool ready = !need || dep_wait(wctx, s, dr, false);
            if (ready || reorder) issue_B(cur ^ 1u, kt + 1); else pend_b = true;
            if (ready) issue_A(cur ^ 1u, kt + 1); else pend_a = true;
        }

        const char* la = lds + cur * Cfg::STAGE_BYTES;
        const char* lb = la + Cfg::A_BYTES;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            V8 af[FM], bf[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) af[i] = *(const V8*)(la + aoff[kk] + i * (32 * 128));
#pragma unroll
            for (int j = 0; j < FN; ++j) bf[j] = *(const V8*)(lb + boff[kk] + j * (32 * 128));
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) acc[i][j] = M::mma(af[i], bf[j], acc[i][j]);
        }

        if (pend_a) {   // the producer was not ready: now really wait, then request the slice
            dep_wait(wctx, s, dr, true);
            if (pend_b) issue_B(cur ^ 1u, kt + 1);
            issue_A(cur ^ 1u, kt + 1);
        }
    }

    // ---- epilogue: activation, round to 16 bits, store ----
    // Accumulator layout of the 32x32 block: lane holds column (lane % 32) and rows
    // 8*(v/4) + 4*(lane/32) + v%4 for v = 0..15.
    if (wctx.ok) {
        T* Cp = (T*)s.C;
        const uint32_t colw = lane & 31u, rowh = (lane >> 5) * 4u;
        if (gate_up) {
            if constexpr (FN >= 2) {
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int jp = 0; jp < FN / 2; ++jp) {
                        const uint32_t col = n0 + (wn * Cfg::WTN) / 2 + jp * 32 + colw;
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const uint32_t row = m0 + wm * Cfg::WTM + i * 32 + 8 * (v / 4) + rowh + (v % 4);
                            const float g = acc[i][2 * jp][v], u = acc[i][2 * jp + 1][v];
                            if (row < s.M && col < s.N) Cp[(size_t)row * s.ldc + col] = (T)(silu_f(g) * u);
                        }
                    }
            }
        } else {
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    const uint32_t col = n0 + wn * Cfg::WTN + j * 32 + colw;
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const uint32_t row = m0 + wm * Cfg::WTM + i * 32 + 8 * (v / 4) + rowh + (v % 4);
                        float x = acc[i][j][v];
                        if (s.act == ACT_GELU) x = gelu_erf(x);
                        else if (s.act == ACT_RELU) x = fmaxf(x, 0.0f);
                        if (row < s.M && col < s.N) Cp[(size_t)row * s.ldc + col] = (T)x;
                    }
                }
        }
    }

    if (SYNC) post_tile(args, s, tile_lin, tx, ty);
}

}  // namespace depsync
