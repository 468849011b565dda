// Peak calibration kernels: what this chip actually sustains, to report next to the published peaks
// (the paper's appendix "A note on MFU" calibrates its own peaks with a large-matmul micro-benchmark).
//   - a register-only loop of v_mfma_f32_16x16x128_f8f6f4 in the 8 x 8 block pattern of the GEMM's wave tile, with
//     operand registers holding either constants or random FP8 bits: the matrix cores are power-limited,
//     and random bits (like real quantized data) sustain a lower clock than constants do;
//   - a 16-bytes-per-lane copy for the HBM read+write rate.
#include "llmq_device.h"
#include "llmq_kernels.h"

namespace llmq {

__device__ inline unsigned mix32(unsigned x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

template <int FA, int FB>
__global__ __launch_bounds__(256, 1) void calibrate_mfma_kernel(float* sink, int iters, int random_bits) {
    v8i a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const unsigned ra = mix32(threadIdx.x * 64 + i * 8 + e + blockIdx.x * 7919u), rb = mix32(ra + 12345u);
            // random sign, exponent and mantissa with the top exponent bit cleared (no NaN / Inf codes)
            a[i][e] = random_bits ? (int)(ra & 0xBFBFBFBFu) : 0x38383838;
            b[i][e] = random_bits ? (int)(rb & 0xBFBFBFBFu) : 0x38383838;
        }
    v4f acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b[j], a[i], acc[i][j], FB, FA, 0, 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) s += acc[i][j][0] + acc[i][j][3];
    if (s == 12345.678f) sink[0] = s;            // keeps the loop alive; practically never taken
}

// 16 KB per workgroup, four 16-byte streaming loads in flight per lane: the fastest of the variants tried on
// this chip (5.9 TB/s; eight or sixteen loads per lane, plain loads, streaming stores and a grid-stride loop
// were all slower, 5.3-5.5 TB/s; hipMemcpy device-to-device 4.9).
__global__ __launch_bounds__(256) void calibrate_copy_kernel(const v4u* __restrict__ src, v4u* __restrict__ dst,
                                                              size_t n_vec) {
    const size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x;
    v4u r[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        r[j] = base + j * 256 < n_vec ? __builtin_nontemporal_load(src + base + j * 256) : v4u{0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (base + j * 256 < n_vec) dst[base + j * 256] = r[j];
}

int launch_calibrate_mfma(int fmtA, int fmtB, int random_bits, int iters, float* d_sink, hipStream_t stream,
                          int num_cus) {
    dim3 grid(num_cus), block(256);
    if (fmtA == 0 && fmtB == 0) hipLaunchKernelGGL((calibrate_mfma_kernel<0, 0>), grid, block, 0, stream, d_sink, iters, random_bits);
    else if (fmtA == 1 && fmtB == 0) hipLaunchKernelGGL((calibrate_mfma_kernel<1, 0>), grid, block, 0, stream, d_sink, iters, random_bits);
    else if (fmtA == 0 && fmtB == 1) hipLaunchKernelGGL((calibrate_mfma_kernel<0, 1>), grid, block, 0, stream, d_sink, iters, random_bits);
    else hipLaunchKernelGGL((calibrate_mfma_kernel<1, 1>), grid, block, 0, stream, d_sink, iters, random_bits);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

int launch_calibrate_copy(const void* src, void* dst, size_t bytes, hipStream_t stream) {
    const size_t n_vec = bytes / 16;
    const size_t blocks = (n_vec + 1023) / 1024;
    hipLaunchKernelGGL(calibrate_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                       reinterpret_cast<const v4u*>(src), reinterpret_cast<v4u*>(dst), n_vec);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace llmq
