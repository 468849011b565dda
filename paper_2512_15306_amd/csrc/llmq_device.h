// Device-side helpers shared by the gfx950 kernels of the FP8 linear path.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace llmq {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned short v2us __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

__host__ __device__ inline float fp8_max(int fmt) { return fmt == 0 ? 448.0f : 57344.0f; }

// Maximum over the 64 lanes of a wavefront: butterfly inside each row of 16 lanes with DPP
// (quad permutes, then the two row mirrors), then the four row results are combined.
__device__ inline unsigned wave_max_u32(unsigned v) {
    unsigned t;
    t = (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
    v = v > t ? v : t;
    t = (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false);   // quad_perm [2,3,0,1]
    v = v > t ? v : t;
    t = (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, false);  // row_half_mirror
    v = v > t ? v : t;
    t = (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, false);  // row_mirror
    v = v > t ? v : t;
    unsigned a = (unsigned)__builtin_amdgcn_readlane((int)v, 0);
    unsigned b = (unsigned)__builtin_amdgcn_readlane((int)v, 16);
    unsigned c = (unsigned)__builtin_amdgcn_readlane((int)v, 32);
    unsigned d = (unsigned)__builtin_amdgcn_readlane((int)v, 48);
    a = a > b ? a : b;
    c = c > d ? c : d;
    return a > c ? a : c;
}

// Magnitude bits of a BF16 absmax -> binary32 bit pattern, NaNs made canonical.
// Non-negative floats order like their bit patterns, so the integer max of these is the float max,
// with NaN (0x7FC00000) above +Inf (0x7F800000) above every finite value.
__device__ inline unsigned amax_bits_from_bf16_mag(unsigned mag16) {
    return mag16 > 0x7F80u ? 0x7FC00000u : (mag16 << 16);
}

}  // namespace llmq
