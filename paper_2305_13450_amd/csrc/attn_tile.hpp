// Middle stage of the attention chain (Fig. 2b of the paper, prompt phase: no cached keys or
// values, dropout is the identity): one tile computes, for one head and one block of 128 query
// rows of one sequence,  T = softmax(Q K^T / sqrt(d) + causal mask) V  with d = 128,
// flash-attention style (keys/values streamed in blocks of 64, running maximum and sum).
//
// MFMA formulation.  Everything is computed transposed so that a lane owns ONE query:
//   S^T[key][q] = K[key][:] . Q[q][:]      A operand = K block (LDS), B operand = Q (registers)
//   O^T[d][q]  += V^T[d][key] P^T[key][q]   A operand = V^T block (LDS), B operand = P^T, which
// is exactly what the S^T accumulators hold: for v_mfma_f32_32x32x16 a lane owns column
// (lane % 32) and rows 8*(v/4) + 4*(lane/32) + v%4, so the 8 accumulator values v0..v0+7 of a
// lane are 8 keys of its query, and since the order of the 16 K-slots of an MFMA is free as
// long as both operands agree, they can be fed straight back as the B operand while V^T is
// read with the same key permutation.  Row maxima and sums are then in-lane reductions plus
// one exchange between the two half-waves.
//
// Dependencies: the tile reads the Q columns of its own rows and the K and V columns of all
// rows of its sequence up to its last row, from the QKV GeMM before it; it posts like any
// producer tile (grid: x = head, y = query block) for the output GeMM after it.
#pragma once
#include <hip/hip_runtime.h>

#include "chain_args.h"
#include "gemm_tile.hpp"
#include "sync_device.hpp"

namespace depsync {

constexpr int ATT_BQ = 128;      // query rows per tile (32 per wave)
constexpr int ATT_BK = 64;       // keys per block
constexpr int ATT_D = 128;       // head dimension
constexpr int ATT_BLK_BYTES = ATT_BK * ATT_D * 2;       // one block of K or V rows (16 KB)
constexpr int ATT_LDS_BYTES = 4 * ATT_BLK_BYTES;        // two K buffers, raw V rows, V^T

// Wait for everything an attention tile reads from the QKV GeMM: producer row tiles y0..y1,
// and in each the column tiles holding this head's Q, K and V columns.
template <bool SYNC>
__device__ __forceinline__ void attn_wait_qkv(WaitCtx& w, const StageDesc& s, uint32_t head, uint32_t row_first,
                                              uint32_t row_last) {
    if (!SYNC || s.dep_kind == DEP_NONE) return;
    const uint32_t E = s.heads * ATT_D;
    const uint32_t y0 = row_first / s.prod_tm, y1 = row_last / s.prod_tm;
    const uint32_t target = s.sem_target_base + s.sem_value;
    for (uint32_t y = y0; y <= y1; ++y) {
        if (s.dep_kind == DEP_ROW) {
            const uint32_t* sem = s.sems + y * SYNC_WORD_STRIDE;
            uint32_t v = sem_load(sem);
            const bool polled = !sem_reached(v, target);
            if (polled) sem_wait(w, sem, target, v);
            count_wait(*w.args, polled);
            continue;
        }
        const uint32_t nblk = (s.dep_kind == DEP_STRIDED) ? 1u : 3u;   // strided: Q, K, V share a semaphore
        for (uint32_t b = 0; b < nblk; ++b) {
            const uint32_t c0 = b * E + head * ATT_D;
            for (uint32_t x = c0 / s.prod_tn; x <= (c0 + ATT_D - 1) / s.prod_tn; ++x) {
                const uint32_t* sem = s.sems + policy_sem(s.dep_kind, x, y, s.prod_grid_y, s.stride) * SYNC_WORD_STRIDE;
                uint32_t v = sem_load(sem);
                const bool polled = !sem_reached(v, target);
                if (polled) sem_wait(w, sem, target, v);
                count_wait(*w.args, polled);
            }
        }
    }
}

// Floats one part of a tile split along the keys leaves in the scratch buffer: the un-normalised
// O^T accumulators of the 256 lanes (64 each), then every lane's running maximum and sum.
constexpr uint32_t ATT_PART_FLOATS = 256 * 64 + 2 * 256;
// Key blocks per part when a tile's keys are split over workgroups (at least this many: a part
// re-reads the queries and leaves 65 KB of partial results).
constexpr uint32_t ATT_MIN_PART_BLOCKS = 4;

template <typename T, bool SYNC, class DR>
__device__ __forceinline__ void attn_tile(const ChainArgs& args, const StageDesc& s, uint32_t head, uint32_t tyz,
                                          uint32_t rel_ticket, char* lds, uint64_t t_enter, DR& dr) {
    using M = Mma<T>;
    using V8 = typename M::V8;
    typedef T T4 __attribute__((ext_vector_type(4)));

    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = uni(tid >> 6);
    const uint32_t h2 = lane >> 5, lq = lane & 31u;
    const uint32_t seq = uni(s.seq), heads = uni(s.heads);
    const uint32_t E = heads * ATT_D;
    const uint32_t ld = uni(s.lda), ldt = uni(s.ldc);
    // A long causal tile is one dependent chain of key blocks, so the stage may split every tile's
    // keys over KS workgroups (the stage's split, as for the GeMM tiles): part z takes a run of
    // whole key blocks, leaves un-normalised results, maxima and sums in the scratch buffer and
    // counts itself in; the last part to arrive combines the parts in key order, normalises,
    // stores and posts.  Tiles of few key blocks use fewer parts (the rest find nothing to do).
    const uint32_t KS = uni(s.ksplit);
    const uint32_t qblk = tyz / KS, part = tyz % KS;
    const uint32_t qblocks = (seq + ATT_BQ - 1) / ATT_BQ;
    const uint32_t b = qblk / qblocks, qb = qblk % qblocks;      // sequence, query block inside it
    const uint32_t seq_row0 = b * seq;                            // first row of the sequence
    const uint32_t q0 = qb * ATT_BQ;                              // first query (inside the sequence)
    const uint32_t q_last = min(q0 + ATT_BQ, seq) - 1;
    const T* QKV = (const T*)uni_ptr(s.A);
    T* Tout = (T*)uni_ptr(s.C);
    // cached keys and values of this sequence come first in key order (token generation)
    const uint32_t cached = uni(s.cached), ldkv = uni(s.ld_cache);
    const T* Kc = (const T*)uni_ptr(s.kcache);
    const T* Vc = (const T*)uni_ptr(s.vcache);

    WaitCtx wctx{&args, rel_ticket, true};
    const bool tracing = SYNC && (args.flags & DS_FLAG_TRACE) && args.trace != nullptr && rel_ticket < args.trace_cap;
    uint64_t t_start = 0, t_ready = 0;
    if (tracing) t_start = now_ticks();

    const uint32_t nblk = (cached + q_last) / ATT_BK + 1;         // key blocks the tile touches
    const uint32_t chunk = max((nblk + KS - 1) / KS, ATT_MIN_PART_BLOCKS);   // key blocks per part
    const uint32_t nparts = (nblk + chunk - 1) / chunk;           // parts that have any (<= KS)
    const uint32_t kb_begin = part * chunk, kb_end = min(nblk, kb_begin + chunk);
    if (part >= nparts) {                                          // nothing for this part: the tile is short
        if (tracing && tid == 0) {
            TraceRec r;
            r.rel = rel_ticket; r.where = hw_where(2u); r.tx = head; r.ty = tyz;
            r.t_enter = t_enter; r.t_start = t_start; r.t_ready = t_start; r.t_end = now_ticks();
            args.trace[rel_ticket] = r;
        }
        return;
    }

    attn_wait_qkv<SYNC>(wctx, s, head, seq_row0, seq_row0 + q_last);
    if (tracing) t_ready = now_ticks();

    // ---- this lane's query row as the B operand of S^T = K Q^T: 8 fragments of 8 d values ----
    const uint32_t qi = q0 + wave * 32 + lq;                      // query index inside the sequence
    const uint32_t qrow = seq_row0 + min(qi, seq - 1);
    V8 qf[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
        qf[kk] = *(const V8*)(QKV + (size_t)qrow * ld + head * ATT_D + kk * 16 + h2 * 8);

    f32x16 o[4];                                                   // O^T: 4 blocks of 32 d x this lane's query
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[i][v] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;
    const float sc = 0.08838834764831845f * 1.4426950408889634f;   // 1/sqrt(128) * log2(e)

    // LDS: two K buffers [64 keys][128 d] (16-byte chunks swizzled by key & 15), one buffer of
    // V rows in the same layout and the V^T block [128 d][64 keys] (8-byte chunks swizzled by d & 15).
    // While block kb is used, the K and V rows of block kb+1 are DMA'd into LDS (no registers
    // held); V is transposed LDS to LDS at the top of the next iteration.
    const uint32_t wave_q_last = min(q0 + wave * 32 + 31, seq - 1);
    char* const ldsVraw = lds + 2 * ATT_BLK_BYTES;
    char* const ldsV = lds + 3 * ATT_BLK_BYTES;
    auto fetch = [&](uint32_t kb) __attribute__((always_inline)) {
        const uint32_t k0 = kb * ATT_BK;
        char* ldsKn = lds + (kb & 1u) * ATT_BLK_BYTES;
#pragma unroll
        for (int i = 0; i < 4; ++i) {                             // 4 x 16 bytes per lane for K, and for V
            const uint32_t idx = i * 256 + tid, row = idx >> 4, slot = idx & 15u, chunk = slot ^ (row & 15u);
            const uint32_t key = k0 + row;                        // position in key order: cache first
            const char *gk, *gv;
            if (key < cached) {
                const size_t r = ((size_t)b * cached + key) * ldkv + head * ATT_D;
                gk = (const char*)(Kc + r); gv = (const char*)(Vc + r);
            } else {
                const uint32_t krow = seq_row0 + min(key - cached, seq - 1);
                gk = (const char*)(QKV + (size_t)krow * ld + E + head * ATT_D);
                gv = gk + E * 2;
            }
            dma16(gk + chunk * 16, ldsKn + (i * 256 + wave * 64) * 16);
            dma16(gv + chunk * 16, ldsVraw + (i * 256 + wave * 64) * 16);   // V rows, same swizzle
        }
    };
    fetch(kb_begin);

    for (uint32_t kb = kb_begin; kb < kb_end; ++kb) {
        const uint32_t k0 = kb * ATT_BK;
        char* ldsK = lds + (kb & 1u) * ATT_BLK_BYTES;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // this wave's part of block kb has landed
        __syncthreads();   // block kb's rows are in LDS for everyone; everyone is done with block kb-1
        // V transposed, LDS to LDS: each lane takes 8 d values of one key, four times
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t idx = i * 256 + tid, key = idx & 63u, dch = idx >> 6;      // dch: 8-wide d chunk 0..15
            const V8 vv = *(const V8*)(ldsVraw + key * 256u + ((dch ^ (key & 15u)) << 4));
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t d = dch * 8 + e;
                const uint32_t off = d * 128u + ((((key >> 2) ^ (d & 15u)) << 3) | ((key & 3u) << 1));
                *(T*)(ldsV + off) = vv[e];
            }
        }
        __syncthreads();   // V^T complete; the raw V rows and the other K buffer are free again
        if (kb + 1 < kb_end) fetch(kb + 1);

        if (k0 <= cached + wave_q_last) {   // blocks entirely above this wave's diagonal contribute nothing
            // ---- S^T for the two 32-key halves of the block ----
            f32x16 st[2];
#pragma unroll
            for (int kh = 0; kh < 2; ++kh) {
#pragma unroll
                for (int v = 0; v < 16; ++v) st[kh][v] = 0.0f;
                const uint32_t row = kh * 32 + lq;
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) {
                    const uint32_t chunk = (kk * 2 + h2) ^ (row & 15u);
                    const V8 kf = *(const V8*)(ldsK + row * 256u + chunk * 16u);
                    st[kh] = M::mma(kf, qf[kk], st[kh]);
                }
            }
            // ---- causal mask, running maximum ----
            float mx = -INFINITY;
#pragma unroll
            for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const uint32_t key = k0 + kh * 32 + 8 * (v / 4) + 4 * h2 + (v % 4);
                    float x = st[kh][v] * sc;
                    if (key > cached + qi || key >= cached + seq) x = -INFINITY;
                    st[kh][v] = x;
                    mx = fmaxf(mx, x);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run, mx);
            // a query beyond the sequence end or with no visible key yet keeps m = -inf: guard the exps
            const float m_use = (m_new == -INFINITY) ? 0.0f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);   // arguments are <= 0 or -inf: v_exp_f32 as is
            float psum = 0.0f;
#pragma unroll
            for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float p = __builtin_amdgcn_exp2f(st[kh][v] - m_use);
                    st[kh][v] = p;
                    psum += p;
                }
            psum += __shfl_xor(psum, 32);
            l_run = l_run * alpha + psum;
            m_run = m_new;
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {   // no query of the wave has a new maximum: O stays
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o[i][v] *= alpha;
            }
            // ---- O^T += V^T P^T : 4 steps of 16 keys ----
#pragma unroll
            for (int step = 0; step < 4; ++step) {
                const int kh = step >> 1, v0 = (step & 1) * 8;
                V8 pf;
#pragma unroll
                for (int j = 0; j < 8; ++j) pf[j] = (T)st[kh][v0 + j];
                const uint32_t kbase = kh * 32 + (step & 1) * 16;          // keys kbase+4h..+3 and kbase+8+4h..+3
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    const uint32_t d = db * 32 + lq;
                    const uint32_t c0 = ((kbase >> 2) + h2) ^ (d & 15u), c1 = ((kbase >> 2) + 2 + h2) ^ (d & 15u);
                    const T4 lo = *(const T4*)(ldsV + d * 128u + (c0 << 3));
                    const T4 hi = *(const T4*)(ldsV + d * 128u + (c1 << 3));
                    V8 vf;
#pragma unroll
                    for (int j = 0; j < 4; ++j) { vf[j] = lo[j]; vf[4 + j] = hi[j]; }
                    o[db] = M::mma(vf, pf, o[db]);
                }
            }
        }
    }

    dr.peek();   // the look at the dispatch queues for the next tile travels while the result is stored
    // ---- keys split over several workgroups: leave the part, carry on only as the last to arrive ----
    bool finish = true;
    if (nparts > 1) {
        const uint32_t tile_lin = qblk * heads + head;
        float* const parts = s.partials + (size_t)tile_lin * KS * ATT_PART_FLOATS;
        float* const mine = parts + (size_t)part * ATT_PART_FLOATS;
        // fragment order, 16 bytes per lane next to its neighbours', written through to memory so
        // that the count below can follow
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                typedef float f32x2 __attribute__((ext_vector_type(2)));
                const f32x2 v2 = {o[i][2 * q], o[i][2 * q + 1]};
                uint64_t bits;
                __builtin_memcpy(&bits, &v2, 8);
                __hip_atomic_store(reinterpret_cast<uint64_t*>(mine + (((i * 8 + q) * 256 + tid) << 1)), bits, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
        __hip_atomic_store(mine + 256 * 64 + 2 * tid, m_run, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(mine + 256 * 64 + 2 * tid + 1, l_run, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();                                           // every wave's part is in memory; the K and V buffers are done with
        uint32_t* flag = reinterpret_cast<uint32_t*>(lds);
        if (tid == 0) {
            const uint32_t old = __hip_atomic_fetch_add(s.arrive + tile_lin * SYNC_WORD_STRIDE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            flag[0] = old;
        }
        __syncthreads();
        finish = __builtin_amdgcn_readfirstlane(flag[0]) == nparts - 1;
        __syncthreads();
        if (finish) {
            // every part is in memory (each counted after its stores had completed): combine in key
            // order, whoever came last, so that the result does not depend on the arrival order
            if (tid == 0) __hip_atomic_store(s.arrive + tile_lin * SYNC_WORD_STRIDE, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            float m_all = -INFINITY;
            for (uint32_t z = 0; z < nparts; ++z)
                m_all = fmaxf(m_all, __hip_atomic_load(parts + (size_t)z * ATT_PART_FLOATS + 256 * 64 + 2 * tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            const float m_use = (m_all == -INFINITY) ? 0.0f : m_all;
            l_run = 0.0f;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[i][v] = 0.0f;
            for (uint32_t z = 0; z < nparts; ++z) {
                const float* pz = parts + (size_t)z * ATT_PART_FLOATS;
                const float mz = __hip_atomic_load(pz + 256 * 64 + 2 * tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const float lz = __hip_atomic_load(pz + 256 * 64 + 2 * tid + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const float g = (mz == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(mz - m_use);
                l_run += lz * g;
                uint64_t t2[32];                                   // agent-scope loads: what the parts wrote through, not a cached line
#pragma unroll
                for (int j = 0; j < 32; ++j)
                    t2[j] = __hip_atomic_load(reinterpret_cast<const uint64_t*>(pz + ((j * 256 + tid) << 1)), __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        typedef float f32x2 __attribute__((ext_vector_type(2)));
                        f32x2 v2;
                        __builtin_memcpy(&v2, &t2[i * 8 + q], 8);
                        o[i][2 * q] += v2[0] * g;
                        o[i][2 * q + 1] += v2[1] * g;
                    }
            }
        }
    }
    // ---- normalise and store: lane owns query qi, d = 32*db + 8*(v/4) + 4*h2 + v%4 ----
    if (finish && wctx.ok && qi < seq) {
        const float inv = 1.0f / l_run;
        T* out = Tout + (size_t)(seq_row0 + qi) * ldt + head * ATT_D;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                T4 pk;
#pragma unroll
                for (int j = 0; j < 4; ++j) pk[j] = (T)(o[db][g * 4 + j] * inv);
                if constexpr (SYNC) {   // written through to memory, like the GeMM tile's output
                    uint64_t bits;
                    __builtin_memcpy(&bits, &pk, 8);
                    __hip_atomic_store(reinterpret_cast<uint64_t*>(out + db * 32 + g * 8 + h2 * 4), bits, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    *(T4*)(out + db * 32 + g * 8 + h2 * 4) = pk;
                }
            }
    }

    dr.grab();   // the increment for the next tile travels while the stores drain
    if (SYNC && finish) post_tile<true>(args, s, qblk * heads + head, head, qblk);
    if (tracing && tid == 0) {
        TraceRec r;
        r.rel = rel_ticket; r.where = hw_where(2u); r.tx = head; r.ty = tyz;
        r.t_enter = t_enter; r.t_start = t_start; r.t_ready = t_ready; r.t_end = now_ticks();
        args.trace[rel_ticket] = r;
    }
}

}  // namespace depsync
