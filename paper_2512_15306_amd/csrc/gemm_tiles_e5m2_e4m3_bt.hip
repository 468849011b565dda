// The tile kernels for E5M2 x E4M3 operands, B T-major.
#include "gemm_tile.h"

namespace llmq {
template bool launch_chosen_tile<1, 0, false, true>(LLMQ_TILE_LAUNCH_PARAMS);
}  // namespace llmq
