// Attention tile for token generation (Fig. 2b with cached keys and values, one new token per
// sequence): one workgroup per (head, sequence).  There is a single query row, so the work is
// streaming the sequence's cached K and V rows once; the matrix cores have nothing to do here.
//
// The four waves split the keys: in every step a wave takes 16 consecutive keys, four lanes
// per key (each lane owns 32 of the 128 head dimensions, so the four read one 256-byte row of
// K and one of V as contiguous quarters; 32 + 32 values of state per lane keep the tile's
// registers well below those of the GeMM tile it shares a kernel with).  Every lane keeps an
// online softmax of its own keys: running maximum m, sum l and 32 un-normalised output values.  At the end the lanes of
// a wave are brought to the wave's maximum and summed through LDS, then the four waves are
// combined the same way, the result is normalised, rounded and stored.  Key order: the cached
// tokens, then the new token's own key (which the QKV GeMM has just produced, like the query).
//
// A handful of (head, sequence) pairs cannot fill 256 CUs, and one workgroup walking thousands
// of keys is a chain of memory round trips, so the keys of a pair are split over `ksplit`
// workgroups (the stage's split, as for the GeMM tiles): each leaves its un-normalised result,
// maximum and sum in the scratch buffer and counts itself in, and the last to arrive combines
// the parts in key order, normalises, stores and posts.
#pragma once
#include <hip/hip_runtime.h>

#include "attn_tile.hpp"
#include "chain_args.h"
#include "sync_device.hpp"

namespace depsync {

constexpr int DEC_LDS_BYTES = 4 * 64 * 33 * 4 + 4 * 130 * 4;   // per-wave transposition areas + the waves' partial results
static_assert(DEC_LDS_BYTES <= ATT_LDS_BYTES, "the generation tile fits the LDS of the attention tile");

template <typename T, bool SYNC, class DR>
__device__ __forceinline__ void attn_decode_tile(const ChainArgs& args, const StageDesc& s, uint32_t head, uint32_t tyz,
                                                 uint32_t rel_ticket, char* lds, uint64_t t_enter, DR& dr) {
    typedef T T8 __attribute__((ext_vector_type(8)));
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = uni(tid >> 6);
    const uint32_t quarter = lane & 3u, slot = lane >> 2;        // quarter of the head dimensions, key slot in the step
    const uint32_t heads = uni(s.heads), E = heads * ATT_D;
    const uint32_t ld = uni(s.lda), ldt = uni(s.ldc);
    const uint32_t cached = uni(s.cached), ldkv = uni(s.ld_cache);
    const T* QKV = (const T*)uni_ptr(s.A);
    const T* Kc = (const T*)uni_ptr(s.kcache);
    const T* Vc = (const T*)uni_ptr(s.vcache);
    T* Tout = (T*)uni_ptr(s.C);
    const uint32_t KS = uni(s.ksplit);
    const uint32_t b = tyz / KS, ks = tyz % KS;                  // sequence, part of its keys
    const uint32_t row = b;                                      // seq = 1: the sequence's only new row

    WaitCtx wctx{&args, rel_ticket, true};
    const bool tracing = SYNC && (args.flags & DS_FLAG_TRACE) && args.trace != nullptr && rel_ticket < args.trace_cap;
    uint64_t t_start = 0, t_ready = 0;
    if (tracing) t_start = now_ticks();
    attn_wait_qkv<SYNC>(wctx, s, head, row, row);
    if (tracing) t_ready = now_ticks();

    // this lane's quarter of the query, scaled to the base-2 softmax: 32 values
    const float sc = 0.08838834764831845f * 1.4426950408889634f;   // 1/sqrt(128) * log2(e)
    float q[32];
    {
        const T* qp = QKV + (size_t)row * ld + head * ATT_D + quarter * 32;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const T8 v = *(const T8*)(qp + c * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) q[c * 8 + e] = (float)v[e] * sc;
        }
    }
    float o[32];
#pragma unroll
    for (int j = 0; j < 32; ++j) o[j] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    const uint32_t n = cached + 1;                               // keys: the cache, then the new token
    const uint32_t chunk = ((n + KS - 1) / KS + 63u) & ~63u;     // keys per part, whole steps of 64
    const uint32_t k_begin = ks * chunk, k_end = min(n, k_begin + chunk);
    for (uint32_t k0 = k_begin + wave * 16; k0 < k_end; k0 += 64) {
        const uint32_t key = k0 + slot;
        const bool live = key < k_end;
        const uint32_t kk = live ? key : n - 1;
        const T *kp, *vp;
        if (kk < cached) {
            const size_t r = ((size_t)b * cached + kk) * ldkv + head * ATT_D + quarter * 32;
            kp = Kc + r; vp = Vc + r;
        } else {
            kp = QKV + (size_t)row * ld + E + head * ATT_D + quarter * 32;
            vp = kp + E;
        }
        T8 kv[4], vv[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) kv[c] = *(const T8*)(kp + c * 8);
#pragma unroll
        for (int c = 0; c < 4; ++c) vv[c] = *(const T8*)(vp + c * 8);
        float dot = 0.0f;
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int e = 0; e < 8; ++e) dot = __builtin_fmaf(q[c * 8 + e], (float)kv[c][e], dot);
        dot += __shfl_xor(dot, 1);                               // the four quarters: the whole score, in all four lanes
        dot += __shfl_xor(dot, 2);
        const float x = live ? dot : -INFINITY;
        const float m_new = fmaxf(m_run, x);
        const float m_use = (m_new == -INFINITY) ? 0.0f : m_new;  // no live key yet: keep the exponentials finite
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
        const float p = __builtin_amdgcn_exp2f(x - m_use);
        l_run = l_run * alpha + p;
        m_run = m_new;
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int e = 0; e < 8; ++e) o[c * 8 + e] = __builtin_fmaf(p, (float)vv[c][e], o[c * 8 + e] * alpha);
    }

    // ---- the wave's lanes to the wave's maximum, summed through LDS ----
    float m_w = m_run;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) m_w = fmaxf(m_w, __shfl_xor(m_w, d));
    const float m_wu = (m_w == -INFINITY) ? 0.0f : m_w;
    const float f = __builtin_amdgcn_exp2f(m_run - m_wu);         // 0 for lanes that saw no live key
    float l_w = (quarter == 0) ? l_run * f : 0.0f;                // the four lanes of a key hold the same l
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) l_w += __shfl_xor(l_w, d);
    float* const tr = reinterpret_cast<float*>(lds) + wave * (64 * 33);
    float* const part = reinterpret_cast<float*>(lds) + 4 * (64 * 33) + wave * 130;   // [128 values, m, l]
    __syncthreads();                                              // (uniform) the LDS is free: the last tile is done with it
#pragma unroll
    for (int j = 0; j < 32; ++j) tr[lane * 33 + j] = o[j] * f;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");            // this wave's writes are in LDS
    __builtin_amdgcn_wave_barrier();
    // each lane sums two of the 128 dimensions over the 16 key slots: dimension q * 32 + j lives in
    // the lanes 4 * slot + q, at position j
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const uint32_t dim = 2 * lane + e, qd = dim >> 5, jj = dim & 31u;
        float acc = 0.0f;
#pragma unroll
        for (int sl = 0; sl < 16; ++sl) acc += tr[(4 * sl + qd) * 33 + jj];
        part[dim] = acc;
    }
    if (lane == 0) { part[128] = m_w; part[129] = l_w; }
    dr.peek();
    __syncthreads();

    // ---- the four waves combined: thread t < 64 owns dimensions 2t, 2t+1 ----
    const float* const all = reinterpret_cast<const float*>(lds) + 4 * (64 * 33);
    float M = -INFINITY, L = 0.0f, r0 = 0.0f, r1 = 0.0f;
    if (tid < 64) {
#pragma unroll
        for (int w = 0; w < 4; ++w) M = fmaxf(M, all[w * 130 + 128]);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float mw = all[w * 130 + 128];
            const float g = (mw == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(mw - M);
            L += all[w * 130 + 129] * g;
            r0 += all[w * 130 + 2 * tid] * g;
            r1 += all[w * 130 + 2 * tid + 1] * g;
        }
    }
    // ---- keys split over several workgroups: leave the part, carry on only as the last to arrive ----
    bool finish = true;
    if (KS > 1) {
        const uint32_t pair = b * heads + head;
        float* const parts = s.partials + (size_t)pair * KS * 130;
        if (tid < 64) {   // written through to memory, so that the count below can follow
            float* dst = parts + ks * 130;
            __hip_atomic_store(dst + 2 * tid, r0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(dst + 2 * tid + 1, r1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (tid == 0) {
                __hip_atomic_store(dst + 128, M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(dst + 129, L, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        uint32_t* flag = reinterpret_cast<uint32_t*>(lds);        // the transposition areas are done with
        if (tid == 0) {
            const uint32_t old = __hip_atomic_fetch_add(s.arrive + pair * SYNC_WORD_STRIDE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            flag[0] = old;
        }
        __syncthreads();
        finish = __builtin_amdgcn_readfirstlane(flag[0]) == KS - 1;
        __syncthreads();
        if (finish) {
            // every part is in memory (each counted after its stores had completed); combine in key order
            if (tid == 0) __hip_atomic_store(s.arrive + pair * SYNC_WORD_STRIDE, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (tid < 64) {
                M = -INFINITY;
                for (uint32_t z = 0; z < KS; ++z)
                    M = fmaxf(M, __hip_atomic_load(parts + z * 130 + 128, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                L = 0.0f; r0 = 0.0f; r1 = 0.0f;
                for (uint32_t z = 0; z < KS; ++z) {
                    const float* pz = parts + z * 130;
                    const float mz = __hip_atomic_load(pz + 128, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const float g = (mz == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(mz - M);
                    L += __hip_atomic_load(pz + 129, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) * g;
                    r0 += __hip_atomic_load(pz + 2 * tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) * g;
                    r1 += __hip_atomic_load(pz + 2 * tid + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) * g;
                }
            }
        }
    }
    // ---- normalised, rounded and stored ----
    if (finish && tid < 64 && wctx.ok) {
        const float inv = 1.0f / L;
        typedef T T2 __attribute__((ext_vector_type(2)));
        T2 pk;
        pk[0] = (T)(r0 * inv); pk[1] = (T)(r1 * inv);
        T* out = Tout + (size_t)row * ldt + head * ATT_D + 2 * tid;
        if constexpr (SYNC) {   // written through to memory, like every tile that posts
            uint32_t bits;
            __builtin_memcpy(&bits, &pk, 4);
            __hip_atomic_store(reinterpret_cast<uint32_t*>(out), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            *(T2*)out = pk;
        }
    }
    dr.grab();
    if (SYNC && finish) post_tile<true>(args, s, b * heads + head, head, b);
    if (tracing && tid == 0) {
        TraceRec r;
        r.rel = rel_ticket; r.where = hw_where(2u); r.tx = head; r.ty = tyz;
        r.t_enter = t_enter; r.t_start = t_start; r.t_ready = t_ready; r.t_end = now_ticks();
        args.trace[rel_ticket] = r;
    }
}

}  // namespace depsync
