// Absmax + scale of a BF16 tensor (paper Section 3 "Overview": tensor-level absmax scaling).
//
// HBM-bound: 2 bytes read per element, nothing else.  Each lane streams 16-byte vectors, keeps a
// packed 16-bit integer maximum of the magnitude bits (exact: |x| orders like bits & 0x7FFF), the
// wavefront combines with DPP, the block with a small LDS tree, and every block stores its result
// in the caller's workspace.  A second, single-block kernel reduces those partial results and
// writes absmax and scale: an intermediate buffer plus a second kernel instead of atomics, the way
// the paper handles reductions (Section 3 "Reproducibility").  Read-modify-write atomics of many
// blocks on one address serialise at roughly 12 ns each on this chip, and an accumulator that
// atomics could target would need a reset launch of its own, which costs as much as the second
// kernel does.
#include <mutex>

#include "llmq_device.h"
#include "llmq_kernels.h"

namespace llmq {

// Scratch of the entry point that allocates nothing and takes no workspace (llmq_amax_static): the per-block
// partial results live in this file-scope array, 4 KB on every GPU the library runs on, held until the
// process ends.  In host code the array's name is only a handle for the runtime: the device address of the
// current GPU's copy comes from hipGetSymbolAddress, once per device, and that address is what kernels and
// launches get.
static __device__ __align__(256) unsigned amax_static_scratch[kAmaxMaxPartials];
constexpr int kMaxDevices = 64;
static unsigned* g_static_scratch_ptr[kMaxDevices];      // per device; guarded by g_static_scratch_mutex
static std::mutex g_static_scratch_mutex;

// Device address of the current GPU's copy of the static scratch, or nullptr if the runtime refuses.
static unsigned* static_scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
    if (g_static_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(amax_static_scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_static_scratch_ptr[dev] = static_cast<unsigned*>(p);
    }
    return g_static_scratch_ptr[dev];
}

constexpr int kAmaxThreads = 256;
constexpr int kAmaxUnroll = 8;          // 16-byte loads in flight per lane

// partial[b] = largest BF16 magnitude pattern (15 bits) seen by block b
__global__ __launch_bounds__(kAmaxThreads) void amax_partial_kernel(
    const v4u* __restrict__ x, size_t n_vec, const uint16_t* __restrict__ tail, int n_tail,
    unsigned* __restrict__ partial) {
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
    m = block_max_u32<kAmaxThreads>(m, s_part);
    if (threadIdx.x == 0) partial[blockIdx.x] = m;
}

// amax = max over the partial results (NaN made canonical), scale = scale_of_amax(amax, FMAX)
__global__ __launch_bounds__(kAmaxThreads) void amax_final_kernel(
    const unsigned* __restrict__ partial, int n_partial, float* __restrict__ d_amax,
    float* __restrict__ d_scale, float fmax) {
    __shared__ unsigned s_part[kAmaxThreads / kWave];
    unsigned m = 0;
    for (int i = threadIdx.x; i < n_partial; i += kAmaxThreads) {
        unsigned v = partial[i];
        m = m > v ? m : v;
    }
    m = block_max_u32<kAmaxThreads>(m, s_part);
    if (threadIdx.x == 0) {
        const float a = __uint_as_float(amax_bits_from_bf16_mag(m));
        *d_amax = a;
        if (d_scale) *d_scale = scale_of_amax(a, fmax);
    }
}

// The same for many partial results (producers that write one per workgroup of a 2-D grid): 1024 lanes,
// four independent 16-byte loads in flight per lane, so that tens of thousands of words take a few
// memory round trips instead of one per word and lane.
constexpr int kAmaxWideThreads = 1024;
__global__ __launch_bounds__(kAmaxWideThreads) void amax_final_wide_kernel(
    const unsigned* __restrict__ partial, int n_partial, float* __restrict__ d_amax,
    float* __restrict__ d_scale, float fmax) {
    __shared__ unsigned s_part[kAmaxWideThreads / kWave];
    unsigned m = 0;
    const int n_vec = n_partial / 4;
    const v4u* pv = reinterpret_cast<const v4u*>(partial);
    int i = threadIdx.x;
    for (; i + 3 * kAmaxWideThreads < n_vec; i += 4 * kAmaxWideThreads) {
        v4u r[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) r[j] = pv[i + j * kAmaxWideThreads];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            unsigned a = r[j][0] > r[j][1] ? r[j][0] : r[j][1], b = r[j][2] > r[j][3] ? r[j][2] : r[j][3];
            a = a > b ? a : b;
            m = m > a ? m : a;
        }
    }
    for (; i < n_vec; i += kAmaxWideThreads) {
        v4u r = pv[i];
        unsigned a = r[0] > r[1] ? r[0] : r[1], b = r[2] > r[3] ? r[2] : r[3];
        a = a > b ? a : b;
        m = m > a ? m : a;
    }
    if ((int)threadIdx.x < n_partial - 4 * n_vec) {
        unsigned v = partial[4 * n_vec + threadIdx.x];
        m = m > v ? m : v;
    }
    m = block_max_u32<kAmaxWideThreads>(m, s_part);
    if (threadIdx.x == 0) {
        const float a = __uint_as_float(amax_bits_from_bf16_mag(m));
        *d_amax = a;
        if (d_scale) *d_scale = scale_of_amax(a, fmax);
    }
}

__global__ void scale_from_amax_kernel(const float* __restrict__ d_amax, float* __restrict__ d_scale, float fmax) {
    *d_scale = scale_of_amax(*d_amax, fmax);
}

int launch_scale_from_amax(const float* d_amax, int fmt, float* d_scale, hipStream_t stream) {
    hipLaunchKernelGGL(scale_from_amax_kernel, dim3(1), dim3(1), 0, stream, d_amax, d_scale, fp8_max(fmt));
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

int launch_amax_final(const unsigned* partial, int n_partial, int fmt, float* d_amax, float* d_scale,
                      hipStream_t stream) {
    if (n_partial <= kAmaxMaxPartials)
        hipLaunchKernelGGL(amax_final_kernel, dim3(1), dim3(kAmaxThreads), 0, stream, partial, n_partial,
                           d_amax, d_scale, fp8_max(fmt));
    else        // partial is 16-byte aligned in that case (checked by the callers that can get here)
        hipLaunchKernelGGL(amax_final_wide_kernel, dim3(1), dim3(kAmaxWideThreads), 0, stream, partial, n_partial,
                           d_amax, d_scale, fp8_max(fmt));
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

int launch_amax(const void* x, size_t n, int fmt, float* d_amax, float* d_scale, void* ws,
                hipStream_t stream, int num_cus) {
    int blocks = 0;
    if (launch_amax_partial(x, n, reinterpret_cast<unsigned*>(ws), &blocks, stream, num_cus) != 0) return -6;
    return launch_amax_final(reinterpret_cast<unsigned*>(ws), blocks, fmt, d_amax, d_scale, stream);
}

// Every block of the first stage writes its word before the second stage reads it, so nothing in the
// scratch has to start at zero; what the last call left there is simply overwritten.
int launch_amax_static(const void* x, size_t n, int fmt, float* d_amax, float* d_scale, hipStream_t stream,
                       int num_cus) {
    unsigned* scratch = static_scratch_of_current_device();
    if (scratch == nullptr) return -6;
    return launch_amax(x, n, fmt, d_amax, d_scale, scratch, stream, num_cus);
}

int launch_amax_partial(const void* x, size_t n, unsigned* partial, int* n_partial, hipStream_t stream, int num_cus) {
    const size_t n_vec = n / 8;
    const int n_tail = (int)(n % 8);
    const size_t chunk = (size_t)kAmaxThreads * kAmaxUnroll;
    const size_t chunks = n_vec / chunk;
    size_t max_blocks = (size_t)num_cus * 4;
    if (max_blocks > (size_t)kAmaxMaxPartials) max_blocks = kAmaxMaxPartials;
    // every workgroup takes the same number of chunks, give or take one: 1452 chunks are 726 workgroups of
    // two, not 1024 of which 428 take a second one while the others wait
    const size_t trips = (chunks + max_blocks - 1) / max_blocks;
    size_t blocks = trips > 0 ? (chunks + trips - 1) / trips : 1;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(amax_partial_kernel, dim3((unsigned)blocks), dim3(kAmaxThreads), 0, stream,
                       reinterpret_cast<const v4u*>(x), n_vec,
                       reinterpret_cast<const uint16_t*>(x) + n_vec * 8, n_tail, partial);
    *n_partial = (int)blocks;
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace llmq
