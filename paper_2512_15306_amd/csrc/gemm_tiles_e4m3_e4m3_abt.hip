// The tile kernels for E4M3 x E4M3 operands, A and B T-major.
#include "gemm_tile.h"

namespace llmq {
template bool launch_chosen_tile<0, 0, true, true>(LLMQ_TILE_LAUNCH_PARAMS);
}  // namespace llmq
