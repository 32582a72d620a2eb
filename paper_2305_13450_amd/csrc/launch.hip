// Dispatch from (tile, dtype, A mode) to the kernel families, the workspace fill kernel and
// the table of macro-tile shapes.
#include <hip/hip_runtime.h>
#include "launch.h"
#include "sync_device.hpp"

namespace depsync {

// Small fill kernel used to (re)zero the workspace; safe to record into a HIP graph.
__global__ void fill_u32_kernel(uint32_t* p, uint32_t value, uint32_t n) {
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}

// Calibration: nothing but bf16 MFMAs on register operands (eight independent 32x32 accumulator
// blocks per wave, no LDS, no memory traffic in the loop).  What this sustains is what the
// matrix cores can do under the chip's power cap for the given operand values.
typedef __bf16 cal_bf16x8 __attribute__((ext_vector_type(8)));
typedef float cal_f32x16 __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256, 2) void mfma_calibration_kernel(const uint4* src, float* out, int iters) {
    const uint32_t t = blockIdx.x * 256 + threadIdx.x;
    cal_bf16x8 a[4], b[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint4 x = src[(t * 6 + i) & 0xffffu];
        __builtin_memcpy(&a[i], &x, 16);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const uint4 y = src[(t * 6 + 4 + j) & 0xffffu];
        __builtin_memcpy(&b[j], &y, 16);
    }
    cal_f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) sum += acc[i][j][v];
    if (sum == 123.456f) out[t] = sum;          // keeps the loop alive; practically never taken
}

hipError_t launch_mfma_calibration(const void* src, float* out, int n_blocks, int iters, hipStream_t stream) {
    hipLaunchKernelGGL(mfma_calibration_kernel, dim3(n_blocks), dim3(256), 0, stream, static_cast<const uint4*>(src), out, iters);
    return hipGetLastError();
}

hipError_t launch_chain_kernel(int tile, int dtype, uint32_t amode, bool sync, uint32_t n_blocks,
                               hipStream_t stream, const ChainArgs& a) {
    if (n_blocks == 0) return hipSuccess;
    if (amode == A_COPY) return launch_copy(sync, n_blocks, stream, a);
    if (amode == A_CONV3X3)
        return dtype == 0 ? launch_bf16_conv(tile, sync, n_blocks, stream, a)
                          : launch_f16_conv(tile, sync, n_blocks, stream, a);
    // a chain whose middle stage is attention for one new token per sequence runs the kernels that
    // hold the token-generation tile
    if (a.n_stages == 3 && a.st[1].op == OP_ATTN && a.st[1].seq == 1)
        return dtype == 0 ? launch_bf16_gemm_gen(tile, sync, n_blocks, stream, a)
                          : launch_f16_gemm_gen(tile, sync, n_blocks, stream, a);
    if (a.n_stages == 3 && a.st[1].op == OP_ATTN)
        return dtype == 0 ? launch_bf16_gemm_attn(tile, sync, n_blocks, stream, a)
                          : launch_f16_gemm_attn(tile, sync, n_blocks, stream, a);
    return dtype == 0 ? launch_bf16_gemm(tile, sync, n_blocks, stream, a)
                      : launch_f16_gemm(tile, sync, n_blocks, stream, a);
}

// Section III-B: a consumer kernel whose workgroups took every slot before the producer's had
// started would wait for ever; the paper holds the consumer's launch back with a one-thread
// kernel until the producer's thread blocks are on the GPU.  Here the producer's persistent
// workgroups each draw a tile as their first action, so "stage has handed out `want` tiles"
// says that they are resident (or that fewer of them have already done more: either way a
// workgroup that keeps drawing the stage's tiles holds a slot).  Lanes 0..7 read one queue
// counter each; the wave sums what has been drawn in this chain's epoch.
__global__ __launch_bounds__(64) void wait_draws_kernel(const ChainArgs a, uint32_t stage, uint32_t want) {
    const uint32_t lane = threadIdx.x;
    const StageDesc& st = a.st[stage];
    const uint32_t len = lane < 8 ? queue_len(st, lane) : 0u;
    uint32_t spins = 0;
    for (;;) {
        uint32_t drawn = 0;
        if (lane < 8 && len != 0) {
            const uint32_t c = __hip_atomic_load(a.ticket + (8u * stage + lane) * SYNC_WORD_STRIDE, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
            const int32_t i = (int32_t)(c - a.queue_epoch * len);   // (may overshoot for a moment: draws past the end are undone)
            drawn = i < 0 ? 0u : ((uint32_t)i > len ? len : (uint32_t)i);
        }
#pragma unroll
        for (int off = 4; off > 0; off >>= 1) drawn += __shfl_down(drawn, off, 8);
        drawn = __builtin_amdgcn_readfirstlane(drawn);
        if (drawn >= want) return;
        if (a.spin_limit != 0 && ++spins >= a.spin_limit) {
            if (lane == 0) {
                const int prev = __hip_atomic_fetch_add(&a.status->timed_out, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (prev == 0)
                    __hip_atomic_store(&a.status->first_timeout, (int32_t)a.first_ticket[stage], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
            }
            return;
        }
        __builtin_amdgcn_s_sleep(16);
    }
}

hipError_t launch_wait_draws(const ChainArgs& a, uint32_t stage, uint32_t want, hipStream_t stream) {
    hipLaunchKernelGGL(wait_draws_kernel, dim3(1), dim3(64), 0, stream, a, stage, want);
    return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t* p, uint32_t value, uint32_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, p, value, n);
    return hipGetLastError();
}

const TileShape* tile_shape(int tile) {
    static const TileShape shapes[] = {
        {0, 0, 0, 0},
        {256, 256, 1, 128},
        {256, 128, 1, 64},
        {128, 256, 1, 128},
        {128, 128, 2, 64},
        {64, 128, 2, 64},
        {64, 64, 2, 32},
        {256, 192, 1, 96},
        {128, 192, 2, 96},
        {256, 64, 2, 64},
        {64, 64, 1, 32},
        {64, 192, 1, 96},
        {128, 192, 1, 96},
        {128, 128, 1, 64},
    };
    if (tile < 1 || tile > 13) return nullptr;
    return &shapes[tile];
}

}  // namespace depsync
