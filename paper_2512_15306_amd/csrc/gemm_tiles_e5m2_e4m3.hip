// The tile kernels for E5M2 x E4M3 operands, both contraction-contiguous.
#include "gemm_tile.h"

namespace llmq {
template bool launch_chosen_tile<1, 0, false, false>(LLMQ_TILE_LAUNCH_PARAMS);
}  // namespace llmq
