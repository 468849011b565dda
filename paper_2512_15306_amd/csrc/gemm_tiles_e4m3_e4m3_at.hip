// The tile kernels for E4M3 x E4M3 operands, A T-major.
#include "gemm_tile.h"

namespace llmq {
template bool launch_chosen_tile<0, 0, true, false>(LLMQ_TILE_LAUNCH_PARAMS);
}  // namespace llmq
