// Instantiates the chain kernels for element type _Float16, A addressing mode A_DENSE, with the
// prompt-phase attention tile as the middle stage.
#include "chain_kernel.hpp"
#include "launch.h"

namespace depsync {
hipError_t launch_f16_gemm_attn(int tile, bool sync, uint32_t n_blocks, hipStream_t stream, const ChainArgs& a) {
    return launch_family<_Float16, A_DENSE, 1>(tile, sync, n_blocks, stream, a);
}
}  // namespace depsync
