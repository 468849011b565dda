// SwiGLU with the extra outputs the FP8 pipeline wants from a non-linearity (paper Section 3,
// kernel-fusion paragraph: every non-linearity also returns the absmax of its result, so the FP8
// conversion of the next matmul's input needs no reduction pass; Section 3 "Activation checkpointing":
// when the absmax is already known, as in recomputation during backward, the conversion itself is
// fused into the non-linearity).
//
//   GU [M, 2I] BF16: columns [0, I) gate g, columns [I, 2I) up u;   h[m,i] = bf16( silu(g) * u )
//   backward: dGU[m, i] = bf16( dh u sg (1 + g (1 - sg)) ),  dGU[m, I+i] = bf16( dh g sg ),  sg = sigma(g)
//
// HBM-bound (forward 4 B read + 2 B written per element of h, or + 1 B + 1 B when FP8 bytes replace
// h; backward 6 B read + 4 B written).  A lane owns a patch of PR rows x 8 columns, exactly the shape
// of the quantize kernel, so the FP8 mode reuses its register transpose: 16-byte loads of g and u,
// arithmetic in binary32, hardware RNE conversion to BF16, packed 16-bit integer absmax on the
// rounded bits, one partial absmax per workgroup (a second kernel reduces them; no atomics).
//
// The arithmetic is fixed operation by operation (IEEE binary32, nothing contracted beyond the
// fused multiply-adds written out) so that the stored bits can be reproduced anywhere:
//   a = -min(max(g,-100),86); n = rint(a*LOG2E); r = fma(n,-LN2_HI,a); r = fma(n,-LN2_LO,r);
//   p = Horner of 1 + r + r^2/2 + ... + r^6/720; e = p * 2^n; sg = 1 / (1 + e); h = (g*sg)*u.
#include <stdlib.h>

#include "llmq_device.h"
#include "llmq_kernels.h"

#pragma clang fp contract(off)

namespace llmq {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float v2f __attribute__((ext_vector_type(2)));

constexpr int kSwThreads = 256;
constexpr int kSwLanesR = 8;                                     // lanes stacked along rows
constexpr int kSwBlockCols = 8 * (kWave / kSwLanesR) * (kSwThreads / kWave);    // 256 columns per workgroup
constexpr int kSwGenericMaxBlocks = 1024;

__device__ inline float sigmoid_f32(float g) {
    const float a = -__builtin_fminf(__builtin_fmaxf(g, -100.0f), 86.0f);
    const float n = __builtin_rintf(a * 0x1.715476p+0f);
    float r = __builtin_fmaf(n, -0x1.62e430p-1f, a);
    r = __builtin_fmaf(n, 0x1.05c610p-29f, r);
    float p = 0x1.6c16c2p-10f;
    p = __builtin_fmaf(p, r, 0x1.111112p-7f);
    p = __builtin_fmaf(p, r, 0x1.555556p-5f);
    p = __builtin_fmaf(p, r, 0x1.555556p-3f);
    p = __builtin_fmaf(p, r, 0.5f);
    p = __builtin_fmaf(p, r, 1.0f);
    p = __builtin_fmaf(p, r, 1.0f);
    const float e = __builtin_ldexpf(p, (int)n);
    const float d = 1.0f + e;
    return 1.0f / d;                                    // correctly rounded division
}

__device__ inline float swiglu_f32(float g, float u) {
    const float silu = g * sigmoid_f32(g);
    return silu * u;
}

__device__ inline unsigned pack_bf16(float lo, float hi) {
    v2f v = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));   // RNE, low half = first
}

__device__ inline float bf16_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(unsigned w) { return __uint_as_float(w & 0xFFFF0000u); }

// Eight elements: one 16-byte vector of g and of u -> one 16-byte vector of h.
__device__ inline v4u swiglu8(const v4u& g, const v4u& u) {
    v4u o;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        o[j] = pack_bf16(swiglu_f32(bf16_lo(g[j]), bf16_lo(u[j])), swiglu_f32(bf16_hi(g[j]), bf16_hi(u[j])));
    return o;
}

__device__ inline void swiglu_bwd_f32(float d, float g, float u, float& dg, float& du) {
    const float sg = sigmoid_f32(g);
    const float silu = g * sg;
    du = d * silu;
    const float one_minus = 1.0f - sg;
    const float t = __builtin_fmaf(g, one_minus, 1.0f);
    float v = d * u;
    v = v * sg;
    dg = v * t;
}

__device__ inline unsigned fold_max(unsigned m0, unsigned m1, unsigned m2, unsigned m3) {
    m0 = pk_max_mag(pk_max_mag(m0, m1), pk_max_mag(m2, m3));
    return (m0 & 0xFFFFu) > (m0 >> 16) ? (m0 & 0xFFFFu) : (m0 >> 16);
}

// Forward.  PR rows per lane (16 when the transposed FP8 copy is written, else 4).  Optional outputs:
// h (WRITE_H), a per-workgroup absmax (AMAX), FP8 codes with a given scale (QFMT >= 0) and their
// transposed copy (TRANSPOSE).  M % PR == 0 and I % 8 == 0: a patch is all inside or all outside.
template <int PR, bool WRITE_H, bool AMAX, int QFMT, bool TRANSPOSE>
__global__ __launch_bounds__(kSwThreads) void swiglu_fwd_patch_kernel(
    const uint16_t* __restrict__ gu, int64_t M, int64_t I, uint16_t* __restrict__ h,
    unsigned* __restrict__ partial, const float* __restrict__ d_qscale, uint8_t* __restrict__ q,
    uint8_t* __restrict__ qt, unsigned grid_cols) {
    static_assert(!TRANSPOSE || PR == 16, "the register transpose works on 16 x 8 patches");
    __shared__ unsigned s_part[kSwThreads / kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    // consecutive workgroups walk along the columns (measured a few percent faster than down the rows)
    const unsigned brow = blockIdx.x / grid_cols, bcol = blockIdx.x % grid_cols;
    const int64_t r0 = (int64_t)brow * (PR * kSwLanesR) + (lane % kSwLanesR) * PR;
    const int64_t c0 = (int64_t)bcol * kSwBlockCols + wave * (8 * (kWave / kSwLanesR)) + (lane / kSwLanesR) * 8;
    const bool live = r0 < M && c0 < I;
    unsigned mag = 0;
    if (live) {
        const uint16_t* src = gu + r0 * (2 * I) + c0;
        // Rows in groups of at most 8: sixteen 16-byte loads in flight per lane, then the arithmetic and the
        // row-major stores of those rows; only the FP8 words of a row (two registers) live on to the transpose.
        constexpr int kGroup = PR < 8 ? PR : 8;
        float s = 0.0f;
        if constexpr (QFMT >= 0) s = *d_qscale;
        unsigned w[PR][2];
        unsigned m0 = 0, m1 = 0, m2 = 0, m3 = 0;
#pragma unroll
        for (int i0 = 0; i0 < PR; i0 += kGroup) {
            v4u g[kGroup], u[kGroup], o[kGroup];
#pragma unroll
            for (int i = 0; i < kGroup; ++i) {
                g[i] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(src + (int64_t)(i0 + i) * 2 * I));
                u[i] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(src + (int64_t)(i0 + i) * 2 * I + I));
            }
#pragma unroll
            for (int i = 0; i < kGroup; ++i) o[i] = swiglu8(g[i], u[i]);
            if constexpr (WRITE_H) {
                uint16_t* dst = h + (r0 + i0) * I + c0;
#pragma unroll
                for (int i = 0; i < kGroup; ++i) *reinterpret_cast<v4u*>(dst + (int64_t)i * I) = o[i];
            }
            if constexpr (AMAX) {
#pragma unroll
                for (int i = 0; i < kGroup; ++i) {
                    m0 = pk_max_mag(m0, o[i][0]);
                    m1 = pk_max_mag(m1, o[i][1]);
                    m2 = pk_max_mag(m2, o[i][2]);
                    m3 = pk_max_mag(m3, o[i][3]);
                }
            }
            if constexpr (QFMT >= 0) {
#pragma unroll
                for (int i = 0; i < kGroup; ++i) quantize8<QFMT>(o[i], s, w[i0 + i][0], w[i0 + i][1]);
                uint8_t* dq = q + (r0 + i0) * I + c0;
#pragma unroll
                for (int i = 0; i < kGroup; ++i) {
                    v2u v = {w[i0 + i][0], w[i0 + i][1]};
                    *reinterpret_cast<v2u*>(dq + (int64_t)i * I) = v;
                }
            }
            if constexpr (PR > kGroup) __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (AMAX) mag = fold_max(m0, m1, m2, m3);
        if constexpr (QFMT >= 0) {
            if constexpr (TRANSPOSE) {
                // column j of the patch -> 16 consecutive bytes of row (c0 + j) of the transposed tensor
                uint8_t* dt = qt + c0 * M + r0;
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    unsigned col[4][4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        unsigned blk[4] = {w[4 * t][k], w[4 * t + 1][k], w[4 * t + 2][k], w[4 * t + 3][k]};
                        unsigned ot[4];
                        transpose4x4_bytes(blk, ot);
#pragma unroll
                        for (int c = 0; c < 4; ++c) col[c][t] = ot[c];
                    }
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        v4u v = {col[c][0], col[c][1], col[c][2], col[c][3]};
                        *reinterpret_cast<v4u*>(dt + (int64_t)(4 * k + c) * M) = v;
                    }
                }
            }
        }
    }
    if constexpr (AMAX) {
        mag = block_max_u32<kSwThreads>(mag, s_part);
        if (threadIdx.x == 0) partial[blockIdx.x] = mag;
    }
}

// FP8 codes in both layouts for tensors made of whole 128 x 256 tiles (every benchmark shape): the lane geometry
// and the LDS transpose of the quantize kernel's tile variant, so that all four streams (g, u, q, q_t) move in
// full 128-byte lines, and the transposed copy can be written in slabs.  The 16 rows of a patch are loaded and
// converted in two groups of eight (sixteen 16-byte loads in flight per lane).
template <bool WRITE_H, int QFMT>
__global__ __launch_bounds__(kTileThreads) void swiglu_fwd_tile_kernel(
    const uint16_t* __restrict__ gu, int64_t M, int64_t I, uint16_t* __restrict__ h,
    const float* __restrict__ d_qscale, uint8_t* __restrict__ q, uint8_t* __restrict__ qt, unsigned grid_cols,
    int64_t qt_row_stride, int64_t qt_band_stride) {
    __shared__ __attribute__((aligned(16))) uint8_t s_t[kTileLdsBytes];
    const unsigned brow = blockIdx.x / grid_cols, bcol = blockIdx.x - brow * grid_cols;   // along the columns first
    int tr, tc;
    tile_patch_origin(tr, tc);
    const int64_t r0 = (int64_t)brow * kTileRows + tr, c0 = (int64_t)bcol * kTileCols + tc;
    const uint16_t* src = gu + r0 * (2 * I) + c0;
    const float s = *d_qscale;
    constexpr int kGroup = 8;
    unsigned w[kPatchRows][2];
#pragma unroll
    for (int i0 = 0; i0 < kPatchRows; i0 += kGroup) {
        v4u g[kGroup], u[kGroup], o[kGroup];
#pragma unroll
        for (int i = 0; i < kGroup; ++i) {
            g[i] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(src + (int64_t)(i0 + i) * 2 * I));
            u[i] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(src + (int64_t)(i0 + i) * 2 * I + I));
        }
#pragma unroll
        for (int i = 0; i < kGroup; ++i) o[i] = swiglu8(g[i], u[i]);
        if constexpr (WRITE_H) {
            uint16_t* dst = h + (r0 + i0) * I + c0;
#pragma unroll
            for (int i = 0; i < kGroup; ++i) *reinterpret_cast<v4u*>(dst + (int64_t)i * I) = o[i];
        }
#pragma unroll
        for (int i = 0; i < kGroup; ++i) quantize8<QFMT>(o[i], s, w[i0 + i][0], w[i0 + i][1]);
        uint8_t* dq = q + (r0 + i0) * I + c0;
#pragma unroll
        for (int i = 0; i < kGroup; ++i) *reinterpret_cast<v2u*>(dq + (int64_t)i * I) = v2u{w[i0 + i][0], w[i0 + i][1]};
        __builtin_amdgcn_sched_barrier(0);
    }
    tile_stage_transposed(w, tr, tc, s_t);
    __syncthreads();
    tile_write_transposed(s_t, qt + (int64_t)bcol * kTileCols * qt_row_stride + (int64_t)brow * qt_band_stride, qt_row_stride);
}

// Backward: dh [M, I], GU [M, 2I] -> dGU [M, 2I], one partial absmax per workgroup.  M % 4 == 0, I % 8 == 0.
__global__ __launch_bounds__(kSwThreads) void swiglu_bwd_patch_kernel(
    const uint16_t* __restrict__ dh, const uint16_t* __restrict__ gu, int64_t M, int64_t I,
    uint16_t* __restrict__ dgu, unsigned* __restrict__ partial, unsigned grid_cols) {
    constexpr int PR = 4;
    __shared__ unsigned s_part[kSwThreads / kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const unsigned brow = blockIdx.x / grid_cols, bcol = blockIdx.x % grid_cols;
    const int64_t r0 = (int64_t)brow * (PR * kSwLanesR) + (lane % kSwLanesR) * PR;
    const int64_t c0 = (int64_t)bcol * kSwBlockCols + wave * (8 * (kWave / kSwLanesR)) + (lane / kSwLanesR) * 8;
    unsigned mag = 0;
    if (r0 < M && c0 < I) {
        const uint16_t* src = gu + r0 * (2 * I) + c0;
        const uint16_t* sd = dh + r0 * I + c0;
        v4u g[PR], u[PR], d[PR];
#pragma unroll
        for (int i = 0; i < PR; ++i) {
            g[i] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(src + (int64_t)i * 2 * I));
            u[i] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(src + (int64_t)i * 2 * I + I));
            d[i] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(sd + (int64_t)i * I));
        }
        unsigned m0 = 0, m1 = 0, m2 = 0, m3 = 0;
        uint16_t* dst = dgu + r0 * (2 * I) + c0;
#pragma unroll
        for (int i = 0; i < PR; ++i) {
            v4u og, ou;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float dg0, du0, dg1, du1;
                swiglu_bwd_f32(bf16_lo(d[i][j]), bf16_lo(g[i][j]), bf16_lo(u[i][j]), dg0, du0);
                swiglu_bwd_f32(bf16_hi(d[i][j]), bf16_hi(g[i][j]), bf16_hi(u[i][j]), dg1, du1);
                og[j] = pack_bf16(dg0, dg1);
                ou[j] = pack_bf16(du0, du1);
            }
            *reinterpret_cast<v4u*>(dst + (int64_t)i * 2 * I) = og;
            *reinterpret_cast<v4u*>(dst + (int64_t)i * 2 * I + I) = ou;
            m0 = pk_max_mag(pk_max_mag(m0, og[0]), ou[0]);
            m1 = pk_max_mag(pk_max_mag(m1, og[1]), ou[1]);
            m2 = pk_max_mag(pk_max_mag(m2, og[2]), ou[2]);
            m3 = pk_max_mag(pk_max_mag(m3, og[3]), ou[3]);
        }
        mag = fold_max(m0, m1, m2, m3);
    }
    mag = block_max_u32<kSwThreads>(mag, s_part);
    if (threadIdx.x == 0) partial[blockIdx.x] = mag;
}

// Any shape, one element per lane and trip.
template <int QFMT>
__global__ __launch_bounds__(kSwThreads) void swiglu_fwd_generic_kernel(
    const uint16_t* __restrict__ gu, int64_t M, int64_t I, uint16_t* __restrict__ h,
    unsigned* __restrict__ partial, const float* __restrict__ d_qscale, uint8_t* __restrict__ q,
    uint8_t* __restrict__ qt) {
    __shared__ unsigned s_part[kSwThreads / kWave];
    const int64_t n = M * I;
    unsigned mag = 0;
    float s = 0.0f;
    if constexpr (QFMT >= 0) s = *d_qscale;
    for (int64_t idx = (int64_t)blockIdx.x * kSwThreads + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * kSwThreads) {
        const int64_t m = idx / I, i = idx - m * I;
        const float g = __uint_as_float((unsigned)gu[m * 2 * I + i] << 16);
        const float u = __uint_as_float((unsigned)gu[m * 2 * I + I + i] << 16);
        const unsigned bits = pack_bf16(swiglu_f32(g, u), 0.0f) & 0xFFFFu;
        if (h) h[idx] = (uint16_t)bits;
        mag = pk_max_mag(mag, bits);
        if constexpr (QFMT >= 0) {
            const float p = __uint_as_float(bits << 16) * s;
            const unsigned code = cvt_pair<QFMT>(p, p, 0u, false) & 0xFFu;
            q[idx] = (uint8_t)code;
            if (qt) qt[i * M + m] = (uint8_t)code;
        }
    }
    if (partial) {
        mag = block_max_u32<kSwThreads>(mag & 0xFFFFu, s_part);
        if (threadIdx.x == 0) partial[blockIdx.x] = mag;
    }
}

__global__ __launch_bounds__(kSwThreads) void swiglu_bwd_generic_kernel(
    const uint16_t* __restrict__ dh, const uint16_t* __restrict__ gu, int64_t M, int64_t I,
    uint16_t* __restrict__ dgu, unsigned* __restrict__ partial) {
    __shared__ unsigned s_part[kSwThreads / kWave];
    const int64_t n = M * I;
    unsigned mag = 0;
    for (int64_t idx = (int64_t)blockIdx.x * kSwThreads + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * kSwThreads) {
        const int64_t m = idx / I, i = idx - m * I;
        const float g = __uint_as_float((unsigned)gu[m * 2 * I + i] << 16);
        const float u = __uint_as_float((unsigned)gu[m * 2 * I + I + i] << 16);
        const float d = __uint_as_float((unsigned)dh[idx] << 16);
        float dg, du;
        swiglu_bwd_f32(d, g, u, dg, du);
        const unsigned w = pack_bf16(dg, du);
        dgu[m * 2 * I + i] = (uint16_t)(w & 0xFFFFu);
        dgu[m * 2 * I + I + i] = (uint16_t)(w >> 16);
        mag = pk_max_mag(mag, w);
    }
    mag = (mag & 0xFFFFu) > (mag >> 16) ? (mag & 0xFFFFu) : (mag >> 16);
    mag = block_max_u32<kSwThreads>(mag, s_part);
    if (threadIdx.x == 0) partial[blockIdx.x] = mag;
}

static bool patch_ok(int64_t M, int64_t I, int pr) { return M % pr == 0 && I % 8 == 0; }

static int64_t generic_blocks(int64_t M, int64_t I) {
    int64_t b = (M * I + kSwThreads - 1) / kSwThreads;
    return b > kSwGenericMaxBlocks ? kSwGenericMaxBlocks : b;
}

// Workgroups of the absmax-producing launches (forward with h, backward): an upper bound of the partial
// results written, which is what the scratch is sized for.
int64_t swiglu_blocks(int64_t M, int64_t I) {
    if (!patch_ok(M, I, 4)) return generic_blocks(M, I);
    return ((M + 4 * kSwLanesR - 1) / (4 * kSwLanesR)) * ((I + kSwBlockCols - 1) / kSwBlockCols);
}

static int64_t patch_blocks(int64_t M, int64_t I, int pr) {
    return ((M + pr * kSwLanesR - 1) / (pr * kSwLanesR)) * ((I + kSwBlockCols - 1) / kSwBlockCols);
}

template <int PR, bool WRITE_H, bool AMAX, int QFMT, bool TRANSPOSE>
static void launch_fwd_patch(const uint16_t* gu, int64_t M, int64_t I, uint16_t* h, unsigned* partial,
                             const float* d_qscale, uint8_t* q, uint8_t* q_t, hipStream_t stream) {
    const unsigned gr = (unsigned)((M + PR * kSwLanesR - 1) / (PR * kSwLanesR)), gc = (unsigned)((I + kSwBlockCols - 1) / kSwBlockCols);
    hipLaunchKernelGGL((swiglu_fwd_patch_kernel<PR, WRITE_H, AMAX, QFMT, TRANSPOSE>), dim3(gr * gc), dim3(kSwThreads), 0, stream,
                       gu, M, I, h, partial, d_qscale, q, q_t, gc);
}

// LLMQ_FUSED_TILE=0 (tuning override, also read by the RMSNorm recompute launch): the register-only patch kernels
// also for tensors made of whole tiles.
static bool use_tile_kernel() {
    if (const char* e = tuning_env("LLMQ_FUSED_TILE")) return atoi(e) != 0;
    return true;
}

template <int QFMT>
static int launch_fwd_fp8(const uint16_t* gu, int64_t M, int64_t I, uint16_t* h, const float* d_qscale,
                          uint8_t* q, uint8_t* q_t, hipStream_t stream, bool qt_slabs) {
    if (qt_slabs && !(q_t && tile_shape_ok(M, I))) return -2;
    if (q_t && tile_shape_ok(M, I) && (qt_slabs || use_tile_kernel())) {
        const unsigned gr = (unsigned)(M / kTileRows), gc = (unsigned)(I / kTileCols);
        const int64_t row_stride = qt_slabs ? kTileRows : M, band_stride = qt_slabs ? I * kTileRows : kTileRows;
        if (h) hipLaunchKernelGGL((swiglu_fwd_tile_kernel<true, QFMT>), dim3(gr * gc), dim3(kTileThreads), 0, stream, gu, M, I, h, d_qscale, q, q_t, gc, row_stride, band_stride);
        else hipLaunchKernelGGL((swiglu_fwd_tile_kernel<false, QFMT>), dim3(gr * gc), dim3(kTileThreads), 0, stream, gu, M, I, h, d_qscale, q, q_t, gc, row_stride, band_stride);
    } else if (q_t && patch_ok(M, I, 16)) {
        if (h) launch_fwd_patch<16, true, false, QFMT, true>(gu, M, I, h, nullptr, d_qscale, q, q_t, stream);
        else launch_fwd_patch<16, false, false, QFMT, true>(gu, M, I, h, nullptr, d_qscale, q, q_t, stream);
    } else if (!q_t && patch_ok(M, I, 4)) {
        if (h) launch_fwd_patch<4, true, false, QFMT, false>(gu, M, I, h, nullptr, d_qscale, q, q_t, stream);
        else launch_fwd_patch<4, false, false, QFMT, false>(gu, M, I, h, nullptr, d_qscale, q, q_t, stream);
    } else {
        hipLaunchKernelGGL((swiglu_fwd_generic_kernel<QFMT>), dim3((unsigned)generic_blocks(M, I)), dim3(kSwThreads), 0,
                           stream, gu, M, I, h, (unsigned*)nullptr, d_qscale, q, q_t);
    }
    return 0;
}

int launch_swiglu_fwd(const void* gu_, int64_t M, int64_t I, void* h_, unsigned* partial, int amax_fmt,
                      float* d_amax, float* d_scale, const float* d_qscale, int q_fmt, uint8_t* q, uint8_t* q_t,
                      hipStream_t stream, bool qt_slabs) {
    const uint16_t* gu = reinterpret_cast<const uint16_t*>(gu_);
    uint16_t* h = reinterpret_cast<uint16_t*>(h_);
    if (q) {                                   // absmax known: FP8 bytes directly, h optional
        const int st = q_fmt == 0 ? launch_fwd_fp8<0>(gu, M, I, h, d_qscale, q, q_t, stream, qt_slabs)
                                  : launch_fwd_fp8<1>(gu, M, I, h, d_qscale, q, q_t, stream, qt_slabs);
        if (st != 0) return st;
        return hipGetLastError() == hipSuccess ? 0 : -6;
    }
    if (qt_slabs) return -2;
    int64_t n_partial;
    if (patch_ok(M, I, 8)) {                   // 8 rows per lane: more bytes in flight, half the partial results
        launch_fwd_patch<8, true, true, -1, false>(gu, M, I, h, partial, nullptr, nullptr, nullptr, stream);
        n_partial = patch_blocks(M, I, 8);
    } else if (patch_ok(M, I, 4)) {
        launch_fwd_patch<4, true, true, -1, false>(gu, M, I, h, partial, nullptr, nullptr, nullptr, stream);
        n_partial = patch_blocks(M, I, 4);
    } else {
        hipLaunchKernelGGL((swiglu_fwd_generic_kernel<-1>), dim3((unsigned)generic_blocks(M, I)), dim3(kSwThreads), 0,
                           stream, gu, M, I, h, partial, (const float*)nullptr, (uint8_t*)nullptr, (uint8_t*)nullptr);
        n_partial = generic_blocks(M, I);
    }
    if (hipGetLastError() != hipSuccess) return -6;
    return launch_amax_final(partial, (int)n_partial, amax_fmt, d_amax, d_scale, stream);
}

int launch_swiglu_bwd(const void* dh, const void* gu, int64_t M, int64_t I, void* dgu, unsigned* partial,
                      int amax_fmt, float* d_amax, float* d_scale, hipStream_t stream) {
    if (patch_ok(M, I, 4)) {
        const unsigned gr = (unsigned)((M + 4 * kSwLanesR - 1) / (4 * kSwLanesR)), gc = (unsigned)((I + kSwBlockCols - 1) / kSwBlockCols);
        hipLaunchKernelGGL(swiglu_bwd_patch_kernel, dim3(gr * gc), dim3(kSwThreads), 0, stream,
                           reinterpret_cast<const uint16_t*>(dh), reinterpret_cast<const uint16_t*>(gu), M, I,
                           reinterpret_cast<uint16_t*>(dgu), partial, gc);
    } else {
        hipLaunchKernelGGL(swiglu_bwd_generic_kernel, dim3((unsigned)generic_blocks(M, I)), dim3(kSwThreads), 0, stream,
                           reinterpret_cast<const uint16_t*>(dh), reinterpret_cast<const uint16_t*>(gu), M, I,
                           reinterpret_cast<uint16_t*>(dgu), partial);
    }
    if (hipGetLastError() != hipSuccess) return -6;
    return launch_amax_final(partial, (int)swiglu_blocks(M, I), amax_fmt, d_amax, d_scale, stream);
}

}  // namespace llmq
