// Dispatch from (tile, dtype, A mode) to the kernel families, the workspace fill kernel and
// the table of macro-tile shapes.
#include <hip/hip_runtime.h>
#include "launch.h"

namespace depsync {

// Small fill kernel used to (re)zero the workspace; safe to record into a HIP graph.
__global__ void fill_u32_kernel(uint32_t* p, uint32_t value, uint32_t n) {
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}

hipError_t launch_chain_kernel(int tile, int dtype, uint32_t amode, bool sync, uint32_t n_blocks,
                               hipStream_t stream, const ChainArgs& a) {
    if (n_blocks == 0) return hipSuccess;
    if (amode == A_CONV3X3)
        return dtype == 0 ? launch_bf16_conv(tile, sync, n_blocks, stream, a)
                          : launch_f16_conv(tile, sync, n_blocks, stream, a);
    return dtype == 0 ? launch_bf16_gemm(tile, sync, n_blocks, stream, a)
                      : launch_f16_gemm(tile, sync, n_blocks, stream, a);
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
    };
    if (tile < 1 || tile > 10) return nullptr;
    return &shapes[tile];
}

}  // namespace depsync
