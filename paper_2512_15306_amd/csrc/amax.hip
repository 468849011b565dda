// Absmax + scale of a BF16 tensor (paper Section 3 "Overview": tensor-level absmax scaling).
//
// HBM-bound: 2 bytes read per element, nothing else.  Each lane streams 16-byte vectors, keeps a
// packed 16-bit integer maximum of the magnitude bits (exact: |x| orders like bits & 0x7FFF), the
// wavefront combines with DPP, the block with a small LDS tree, and blocks meet in one integer
// atomic max, whose result is order-independent and therefore deterministic.  The last block to
// finish turns the absmax into the scale, so no third launch is needed.
#include "llmq_device.h"
#include "llmq_kernels.h"

namespace llmq {

constexpr int kAmaxThreads = 256;
constexpr int kAmaxUnroll = 8;          // 16-byte loads in flight per lane

__global__ void amax_reset_kernel(unsigned* amax_bits, unsigned* ticket) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        *amax_bits = 0u;
        if (ticket) *ticket = 0u;
    }
}

__device__ inline unsigned pk_max_mag(unsigned acc, unsigned w) {
    v2us a = __builtin_bit_cast(v2us, acc);
    v2us b = __builtin_bit_cast(v2us, w & 0x7FFF7FFFu);
    return __builtin_bit_cast(unsigned, __builtin_elementwise_max(a, b));
}

__global__ __launch_bounds__(kAmaxThreads) void amax_kernel(
    const v4u* __restrict__ x, size_t n_vec, const uint16_t* __restrict__ tail, int n_tail,
    unsigned* __restrict__ amax_bits, unsigned* __restrict__ ticket_then_scale, float fmax) {
    __shared__ unsigned s_part[kAmaxThreads / kWave];
    unsigned m0 = 0, m1 = 0, m2 = 0, m3 = 0;      // packed pairs of 15-bit magnitudes
    const size_t chunk = (size_t)kAmaxThreads * kAmaxUnroll;
    for (size_t base = (size_t)blockIdx.x * chunk; base < n_vec; base += (size_t)gridDim.x * chunk) {
        v4u r[kAmaxUnroll];
#pragma unroll
        for (int j = 0; j < kAmaxUnroll; ++j) {
            size_t i = base + (size_t)j * kAmaxThreads + threadIdx.x;
            r[j] = i < n_vec ? __builtin_nontemporal_load(x + i) : v4u{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int j = 0; j < kAmaxUnroll; ++j) {
            m0 = pk_max_mag(m0, r[j][0]);
            m1 = pk_max_mag(m1, r[j][1]);
            m2 = pk_max_mag(m2, r[j][2]);
            m3 = pk_max_mag(m3, r[j][3]);
        }
    }
    m0 = pk_max_mag(pk_max_mag(m0, m1), pk_max_mag(m2, m3));
    unsigned m = (m0 & 0xFFFFu) > (m0 >> 16) ? (m0 & 0xFFFFu) : (m0 >> 16);
    if (blockIdx.x == 0 && (int)threadIdx.x < n_tail) {          // the n % 8 trailing elements
        unsigned t = tail[threadIdx.x] & 0x7FFFu;
        m = m > t ? m : t;
    }
    m = wave_max_u32(m);
    if ((threadIdx.x & (kWave - 1)) == 0) s_part[threadIdx.x / kWave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kAmaxThreads / kWave; ++w) m = m > s_part[w] ? m : s_part[w];
        atomicMax(amax_bits, amax_bits_from_bf16_mag(m));
        bool last = false;
        if (ticket_then_scale) {
            __threadfence();
            last = atomicAdd(ticket_then_scale, 1u) == gridDim.x - 1;
        }
        if (last) {
            __threadfence();
            unsigned bits = atomicMax(amax_bits, 0u);            // coherent read of the final value
            float a = __uint_as_float(bits);
            float s;
            if (a == 0.0f) {
                s = 1.0f;
            } else {
                s = fmax / a;                                     // one correctly rounded division
                if (__builtin_isinf(s)) s = 3.402823466e+38f;
            }
            *reinterpret_cast<float*>(ticket_then_scale) = s;
        }
    }
}

int launch_amax(const void* x, size_t n, int fmt, float* d_amax, float* d_scale, hipStream_t stream,
                int num_cus) {
    const size_t n_vec = n / 8;
    const int n_tail = (int)(n % 8);
    const size_t chunk = (size_t)kAmaxThreads * kAmaxUnroll;
    size_t blocks = (n_vec + chunk - 1) / chunk;
    const size_t max_blocks = (size_t)num_cus * 8;
    if (blocks > max_blocks) blocks = max_blocks;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(amax_reset_kernel, dim3(1), dim3(64), 0, stream,
                       reinterpret_cast<unsigned*>(d_amax), reinterpret_cast<unsigned*>(d_scale));
    hipLaunchKernelGGL(amax_kernel, dim3((unsigned)blocks), dim3(kAmaxThreads), 0, stream,
                       reinterpret_cast<const v4u*>(x), n_vec,
                       reinterpret_cast<const uint16_t*>(x) + n_vec * 8, n_tail,
                       reinterpret_cast<unsigned*>(d_amax), reinterpret_cast<unsigned*>(d_scale),
                       fp8_max(fmt));
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace llmq
