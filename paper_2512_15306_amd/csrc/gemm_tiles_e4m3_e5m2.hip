// The tile kernels for E4M3 x E5M2 operands, both contraction-contiguous.
#include "gemm_tile.h"

namespace llmq {
template bool launch_chosen_tile<0, 1, false, false>(LLMQ_TILE_LAUNCH_PARAMS);
}  // namespace llmq
