// Instantiates the chain kernels for element type __bf16, A addressing mode A_DENSE, with the
// token-generation attention tile as the middle stage.
#include "chain_kernel.hpp"
#include "launch.h"

namespace depsync {
hipError_t launch_bf16_gemm_gen(int tile, bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a) {
    return launch_family<__bf16, A_DENSE, 2>(tile, sync, n_blocks, stream, a);
}
}  // namespace depsync
