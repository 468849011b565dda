// Absmax + scale of a BF16 tensor (paper Section 3 "Overview": tensor-level absmax scaling).
//
// HBM-bound: 2 bytes read per element, nothing else.  Each lane streams 16-byte vectors, keeps a
// packed 16-bit integer maximum of the magnitude bits (exact: |x| orders like bits & 0x7FFF), the
// wavefront combines with DPP, the block with a small LDS tree.  Blocks meet in integer atomics:
// max on the absmax bits and min on the scale bits (the scale FMAX/amax falls as amax grows, and
// non-negative floats order like their bit patterns), both order-independent and therefore
// deterministic.  Read-modify-write atomics of many blocks on one address serialise at roughly
// 12 ns each on this chip, so a block first reads the running maximum and only issues its atomics
// when it would raise it; on real tensors that is a handful of blocks.
#include "llmq_device.h"
#include "llmq_kernels.h"

namespace llmq {

constexpr int kAmaxThreads = 256;
constexpr int kAmaxUnroll = 8;          // 16-byte loads in flight per lane

__global__ void amax_reset_kernel(unsigned* amax_bits, unsigned* scale_bits) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        *amax_bits = 0u;
        if (scale_bits) *scale_bits = 0x7F7FFFFFu;       // FLT_MAX: the scale of an all-zero tensor
    }
}

__device__ inline unsigned pk_max_mag(unsigned acc, unsigned w) {
    v2us a = __builtin_bit_cast(v2us, acc);
    v2us b = __builtin_bit_cast(v2us, w & 0x7FFF7FFFu);
    return __builtin_bit_cast(unsigned, __builtin_elementwise_max(a, b));
}

__global__ __launch_bounds__(kAmaxThreads) void amax_kernel(
    const v4u* __restrict__ x, size_t n_vec, const uint16_t* __restrict__ tail, int n_tail,
    unsigned* __restrict__ amax_bits, unsigned* __restrict__ scale_bits, float fmax) {
    __shared__ unsigned s_part[kAmaxThreads / kWave];
    unsigned m0 = 0, m1 = 0, m2 = 0, m3 = 0;      // packed pairs of 15-bit magnitudes
    const size_t chunk = (size_t)kAmaxThreads * kAmaxUnroll;
    const size_t n_full = n_vec / chunk;
    for (size_t c = blockIdx.x; c < n_full; c += gridDim.x) {
        const v4u* p = x + c * chunk + threadIdx.x;
        v4u r[kAmaxUnroll];
#pragma unroll
        for (int j = 0; j < kAmaxUnroll; ++j) r[j] = __builtin_nontemporal_load(p + j * kAmaxThreads);
#pragma unroll
        for (int j = 0; j < kAmaxUnroll; ++j) {
            m0 = pk_max_mag(m0, r[j][0]);
            m1 = pk_max_mag(m1, r[j][1]);
            m2 = pk_max_mag(m2, r[j][2]);
            m3 = pk_max_mag(m3, r[j][3]);
        }
    }
    if (blockIdx.x == gridDim.x - 1) {            // the partial chunk and the n % 8 trailing elements
        for (size_t i = n_full * chunk + threadIdx.x; i < n_vec; i += kAmaxThreads) {
            v4u r = x[i];
            m0 = pk_max_mag(m0, r[0]);
            m1 = pk_max_mag(m1, r[1]);
            m2 = pk_max_mag(m2, r[2]);
            m3 = pk_max_mag(m3, r[3]);
        }
        if ((int)threadIdx.x < n_tail) m0 = pk_max_mag(m0, (unsigned)tail[threadIdx.x]);
    }
    m0 = pk_max_mag(pk_max_mag(m0, m1), pk_max_mag(m2, m3));
    unsigned m = (m0 & 0xFFFFu) > (m0 >> 16) ? (m0 & 0xFFFFu) : (m0 >> 16);
    m = wave_max_u32(m);
    if ((threadIdx.x & (kWave - 1)) == 0) s_part[threadIdx.x / kWave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kAmaxThreads / kWave; ++w) m = m > s_part[w] ? m : s_part[w];
        const unsigned bits = amax_bits_from_bf16_mag(m);
        // A stale value is never above the true running maximum, so skipping on it is safe: whoever
        // wrote that value also issues (or has issued) the matching scale.
        const unsigned cur = __hip_atomic_load(amax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (bits > cur) {
            atomicMax(amax_bits, bits);
            if (scale_bits) {
                float s = fmax / __uint_as_float(bits);           // one correctly rounded division
                if (__builtin_isinf(s)) s = 3.402823466e+38f;
                atomicMin(scale_bits, __float_as_uint(s));        // a NaN scale (NaN absmax) never wins
            }
        }
    }
}

int launch_amax(const void* x, size_t n, int fmt, float* d_amax, float* d_scale, hipStream_t stream,
                int num_cus) {
    const size_t n_vec = n / 8;
    const int n_tail = (int)(n % 8);
    const size_t chunk = (size_t)kAmaxThreads * kAmaxUnroll;
    size_t blocks = n_vec / chunk;
    const size_t max_blocks = (size_t)num_cus * 4;
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
