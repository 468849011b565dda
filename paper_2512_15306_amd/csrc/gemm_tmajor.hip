// FP8 contraction with T-major operands: the backward GEMMs on the untransposed quantized tensors, so that
// no transposed copy has to be written (the paper's Section 3 keeps such copies because its FP8 GEMM only
// takes contraction-contiguous operands; gfx950's transposing LDS reads lift that restriction).
//   B T-major          : dX[m,k] = sum_n dYq[m,n] Wq[n,k]        (A = dYq [M,N], B = Wq [N,K])
//   A and B T-major    : dW[n,k] = sum_m dYq[m,n] Xq[m,k]        (A = dYq [M,N], B = Xq [M,K])
//   A T-major only     : completes the set.
#include "gemm_tile.h"

namespace llmq {

void launch_gemm_generic(const uint8_t* A, int fmtA, int layout_a, const uint8_t* B, int fmtB, int layout_b, int64_t R, int64_t C,
                         int64_t T, const float* sA, const float* sB, void* c, int accumulate, unsigned* amax,
                         hipStream_t stream);
void launch_gemm_amax_reset(unsigned* amax, hipStream_t stream);

template <int FA, int FB>
static bool launch_layout(bool ta, bool tb, const uint8_t* A, const uint8_t* B, int64_t R, int64_t C, int64_t T,
                          const float* sA, const float* sB, void* c, int accumulate, unsigned* amax,
                          hipStream_t stream, int num_cus, GemmScratch scratch, bool slabs_a, bool slabs_b) {
    if (ta && tb) return launch_chosen_tile<FA, FB, true, true>(A, B, R, C, T, sA, sB, c, accumulate, amax, stream, num_cus, scratch, false, false);
    if (tb) return launch_chosen_tile<FA, FB, false, true>(A, B, R, C, T, sA, sB, c, accumulate, amax, stream, num_cus, scratch, slabs_a, false);
    return launch_chosen_tile<FA, FB, true, false>(A, B, R, C, T, sA, sB, c, accumulate, amax, stream, num_cus, scratch, false, slabs_b);
}

int launch_gemm_fp8(const uint8_t* A, int fmtA, int layout_a, const uint8_t* B, int fmtB, int layout_b, int64_t R, int64_t C,
                    int64_t T, const float* d_scaleA, const float* d_scaleB, void* c_bf16, int accumulate,
                    float* d_amax_c, bool amax_is_zeroed, hipStream_t stream, int num_cus, GemmScratch scratch) {
    const bool ta = layout_a == kLayoutTMajor, tb = layout_b == kLayoutTMajor;
    const bool slabs_a = layout_a == kLayoutSlabs, slabs_b = layout_b == kLayoutSlabs;
    if (!ta && !tb)
        return launch_gemm_tn(A, fmtA, B, fmtB, R, C, T, d_scaleA, d_scaleB, c_bf16, accumulate, d_amax_c, amax_is_zeroed, stream, num_cus,
                              scratch, slabs_a, slabs_b);
    unsigned* amax = reinterpret_cast<unsigned*>(d_amax_c);
    if (amax && !amax_is_zeroed) launch_gemm_amax_reset(amax, stream);
    // The tile kernel addresses a T-major operand with 32-bit byte offsets from its first tile column (an operand
    // in slabs from its first tile row) and keeps 0x7FFFFF00 as the offset that is out of range for sure; B is
    // always E4M3 in the tuned set (weights and activations), other mixes take the generic kernel.
    const int64_t lim = 0x7FFFFF00ll - ((int64_t)1 << 24);
    const bool fits = (!(ta || slabs_a) || (T + 256) * R < lim) && (!(tb || slabs_b) || (T + 256) * C < lim);
    bool done = false;
    if (fits && fmtB == 0) {
        if (fmtA == 0) done = launch_layout<0, 0>(ta, tb, A, B, R, C, T, d_scaleA, d_scaleB, c_bf16, accumulate, amax, stream, num_cus, scratch, slabs_a, slabs_b);
        else done = launch_layout<1, 0>(ta, tb, A, B, R, C, T, d_scaleA, d_scaleB, c_bf16, accumulate, amax, stream, num_cus, scratch, slabs_a, slabs_b);
    }
    if (!done) launch_gemm_generic(A, fmtA, layout_a, B, fmtB, layout_b, R, C, T, d_scaleA, d_scaleB, c_bf16, accumulate, amax, stream);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace llmq
