// The tile kernels for E4M3 x E4M3 operands, B T-major.
#include "gemm_tile.h"

namespace llmq {
template bool launch_chosen_tile<0, 0, false, true>(LLMQ_TILE_LAUNCH_PARAMS);
}  // namespace llmq
