// Host-side launchers of the gfx950 kernels (internal to the library; the public ABI is llmq.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace llmq {

// Each returns 0 or LLMQ_ERR_DEVICE (-6).  Arguments are validated by the callers in api.hip.
constexpr int kAmaxMaxPartials = 1024;      // the absmax workspace holds one 32-bit word per block
int launch_amax(const void* x, size_t n, int fmt, float* d_amax, float* d_scale, void* ws,
                hipStream_t stream, int num_cus);
// zero_word: if not NULL, one 32-bit word the kernel also clears (the absmax accumulator of the GEMM
// that follows in the same call, which saves a launch).
int launch_quantize(const void* x, int64_t rows, int64_t cols, const float* d_scale, int fmt,
                    uint8_t* q, uint8_t* q_t, unsigned* zero_word, hipStream_t stream);
int launch_gemm_tn(const uint8_t* A, int fmtA, const uint8_t* B, int fmtB, int64_t R, int64_t C,
                   int64_t T, const float* d_scaleA, const float* d_scaleB, void* c_bf16,
                   int accumulate, float* d_amax_c, bool amax_is_zeroed, hipStream_t stream, int num_cus);

int launch_calibrate_mfma(int fmtA, int fmtB, int random_bits, int iters, float* d_sink, hipStream_t stream,
                          int num_cus);
int launch_calibrate_copy(const void* src, void* dst, size_t bytes, hipStream_t stream);

}  // namespace llmq
