// The tile kernels for BF16 x BF16 (the baseline) operands, both contraction-contiguous.
#include "gemm_tile.h"

namespace llmq {
template bool launch_chosen_tile<kFmtBf16, kFmtBf16, false, false>(LLMQ_TILE_LAUNCH_PARAMS);
}  // namespace llmq
