// RMSNorm joined with the residual addition, with the extra outputs of the FP8 pipeline (paper
// Section 3, kernel-fusion paragraph: RMS-norm and residual-stream addition are one kernel that also
// returns the absmax of the normalised output; Section 3 "Activation checkpointing": with the
// statistics kept from the forward pass, the FP8 conversion is fused in during recomputation).
//
//   res'[m,c] = bf16( res[m,c] + x[m,c] ),  rstd[m] = 1 / sqrt( mean_c res'[m,c]^2 + eps ),
//   y[m,c]    = bf16( (res'[m,c] * rstd[m]) * w[c] )
//
// Forward kernel: one wavefront per row, the row stays in registers between the reduction and the
// normalisation (one pass over HBM: 4 B read, 2 + 2 B written per element; 2 B less without the
// addition), sum of squares in binary32 with a butterfly over the lanes, absmax of y as a packed
// integer max of the rounded bits, one partial absmax per workgroup for the second-stage kernel.
// Recompute kernel: rstd and the scale are inputs, so the operation is element-wise; it has the
// lane geometry of the quantize kernel (16 rows x 8 columns per lane) and reuses its register
// transpose to write the FP8 codes in both layouts (2 B read, 1 + 1 B written per element).
#include <stdlib.h>

#include "llmq_device.h"
#include "llmq_kernels.h"

#pragma clang fp contract(off)

namespace llmq {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float v2f __attribute__((ext_vector_type(2)));

constexpr int kRnThreads = 256;
constexpr int kRnRowsPerBlock = kRnThreads / kWave;        // one wavefront per row
constexpr int kRnMaxVec = 16;                               // 16-byte vectors per lane kept in registers
constexpr int kRnMaxC = kRnMaxVec * kWave * 8;              // 8192 columns

__device__ inline unsigned rn_pack(float lo, float hi) {
    v2f v = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}
__device__ inline float rn_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ inline float rn_hi(unsigned w) { return __uint_as_float(w & 0xFFFF0000u); }

__device__ inline float wave_sum_f32(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ inline unsigned fold_pairs(unsigned m0, unsigned m1, unsigned m2, unsigned m3) {
    m0 = pk_max_mag(pk_max_mag(m0, m1), pk_max_mag(m2, m3));
    return (m0 & 0xFFFFu) > (m0 >> 16) ? (m0 & 0xFFFFu) : (m0 >> 16);
}

// y = bf16((r * rstd) * w) for the eight elements of one 16-byte vector
__device__ inline v4u normalize8(const v4u& r, float rstd, const v4u& w) {
    v4u o;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float a = rn_lo(r[j]) * rstd, b = rn_hi(r[j]) * rstd;
        o[j] = rn_pack(a * rn_lo(w[j]), b * rn_hi(w[j]));
    }
    return o;
}

// C % 8 == 0, C <= 8192.  x == nullptr: no addition (res is normalised as it is, res_out is not written).
template <bool HAS_X>
__global__ __launch_bounds__(kRnThreads) void rmsnorm_row_kernel(
    const uint16_t* res, const uint16_t* __restrict__ x, const uint16_t* __restrict__ w,
    int64_t M, int C, float eps, uint16_t* res_out, uint16_t* __restrict__ y,
    float* __restrict__ rstd_out, unsigned* __restrict__ partial) {
    // res_out may be res (addition in place): every lane reads its elements before it writes them
    __shared__ unsigned s_part[kRnThreads / kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t row = (int64_t)blockIdx.x * kRnRowsPerBlock + wave;
    const int nvec = C / 8;
    unsigned mag = 0;
    if (row < M) {
        const v4u* pr = reinterpret_cast<const v4u*>(res + row * C);
        const v4u* px = HAS_X ? reinterpret_cast<const v4u*>(x + row * C) : nullptr;
        v4u r[kRnMaxVec];
#pragma unroll
        for (int k = 0; k < kRnMaxVec; ++k) {
            const int idx = k * kWave + lane;
            if (k * kWave < nvec && idx < nvec) {
                r[k] = __builtin_nontemporal_load(pr + idx);
                if constexpr (HAS_X) {
                    const v4u xv = __builtin_nontemporal_load(px + idx);
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        r[k][j] = rn_pack(rn_lo(r[k][j]) + rn_lo(xv[j]), rn_hi(r[k][j]) + rn_hi(xv[j]));
                }
            }
        }
        float ss = 0.0f;
#pragma unroll
        for (int k = 0; k < kRnMaxVec; ++k) {
            const int idx = k * kWave + lane;
            if (k * kWave < nvec && idx < nvec) {
                if constexpr (HAS_X) *reinterpret_cast<v4u*>(res_out + row * C + (int64_t)idx * 8) = r[k];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float a = rn_lo(r[k][j]), b = rn_hi(r[k][j]);
                    ss = __builtin_fmaf(a, a, ss);
                    ss = __builtin_fmaf(b, b, ss);
                }
            }
        }
        ss = wave_sum_f32(ss);
        const float ms = ss / (float)C;
        const float rstd = 1.0f / __builtin_sqrtf(ms + eps);
        if (lane == 0) rstd_out[row] = rstd;
        unsigned m0 = 0, m1 = 0, m2 = 0, m3 = 0;
        const v4u* pw = reinterpret_cast<const v4u*>(w);
#pragma unroll
        for (int k = 0; k < kRnMaxVec; ++k) {
            const int idx = k * kWave + lane;
            if (k * kWave < nvec && idx < nvec) {
                const v4u o = normalize8(r[k], rstd, pw[idx]);
                *reinterpret_cast<v4u*>(y + row * C + (int64_t)idx * 8) = o;
                m0 = pk_max_mag(m0, o[0]);
                m1 = pk_max_mag(m1, o[1]);
                m2 = pk_max_mag(m2, o[2]);
                m3 = pk_max_mag(m3, o[3]);
            }
        }
        mag = fold_pairs(m0, m1, m2, m3);
    }
    mag = block_max_u32<kRnThreads>(mag, s_part);
    if (threadIdx.x == 0) partial[blockIdx.x] = mag;
}

// Any C: one wavefront per row, element-wise strided loops; the row is read again for the second pass
// (from res_out when the addition was done).
__global__ __launch_bounds__(kRnThreads) void rmsnorm_row_generic_kernel(
    const uint16_t* res, const uint16_t* __restrict__ x, const uint16_t* __restrict__ w,
    int64_t M, int64_t C, float eps, uint16_t* res_out, uint16_t* __restrict__ y,
    float* __restrict__ rstd_out, unsigned* __restrict__ partial) {
    __shared__ unsigned s_part[kRnThreads / kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t row = (int64_t)blockIdx.x * kRnRowsPerBlock + wave;
    unsigned mag = 0;
    if (row < M) {
        float ss = 0.0f;
        for (int64_t c = lane; c < C; c += kWave) {
            unsigned bits = res[row * C + c];
            if (x) {
                bits = rn_pack(__uint_as_float(bits << 16) + __uint_as_float((unsigned)x[row * C + c] << 16), 0.0f) & 0xFFFFu;
                res_out[row * C + c] = (uint16_t)bits;
            }
            const float v = __uint_as_float(bits << 16);
            ss = __builtin_fmaf(v, v, ss);
        }
        ss = wave_sum_f32(ss);
        const float ms = ss / (float)C;
        const float rstd = 1.0f / __builtin_sqrtf(ms + eps);
        if (lane == 0) rstd_out[row] = rstd;
        const uint16_t* src = x ? res_out : res;          // this lane re-reads exactly the elements it wrote
        for (int64_t c = lane; c < C; c += kWave) {
            const float t = __uint_as_float((unsigned)src[row * C + c] << 16) * rstd;
            const unsigned o = rn_pack(t * __uint_as_float((unsigned)w[c] << 16), 0.0f) & 0xFFFFu;
            y[row * C + c] = (uint16_t)o;
            mag = pk_max_mag(mag, o);
        }
    }
    mag = block_max_u32<kRnThreads>(mag & 0xFFFFu, s_part);
    if (threadIdx.x == 0) partial[blockIdx.x] = mag;
}

// Recompute path: rstd [M] and the scale are given.  Lane = PR rows x 8 columns (PR = 16 with the
// transposed copy, else 4); M % PR == 0, C % 8 == 0.
constexpr int kRnLanesR = 8;
constexpr int kRnBlockCols = 8 * (kWave / kRnLanesR) * (kRnThreads / kWave);

template <int PR, int QFMT, bool TRANSPOSE, bool WRITE_Y>
__global__ __launch_bounds__(kRnThreads) void rmsnorm_apply_fp8_patch_kernel(
    const uint16_t* __restrict__ res, const uint16_t* __restrict__ w, const float* __restrict__ rstd,
    int64_t M, int64_t C, const float* __restrict__ d_qscale, uint8_t* __restrict__ q,
    uint8_t* __restrict__ qt, uint16_t* __restrict__ y, unsigned grid_cols) {
    static_assert(!TRANSPOSE || PR == 16, "the register transpose works on 16 x 8 patches");
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const unsigned brow = blockIdx.x / grid_cols, bcol = blockIdx.x % grid_cols;     // walk along the columns
    const int64_t r0 = (int64_t)brow * (PR * kRnLanesR) + (lane % kRnLanesR) * PR;
    const int64_t c0 = (int64_t)bcol * kRnBlockCols + wave * (8 * (kWave / kRnLanesR)) + (lane / kRnLanesR) * 8;
    if (r0 >= M || c0 >= C) return;
    const uint16_t* src = res + r0 * C + c0;
    v4u in[PR];
#pragma unroll
    for (int i = 0; i < PR; ++i) in[i] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(src + (int64_t)i * C));
    const v4u wv = *reinterpret_cast<const v4u*>(w + c0);
    float rs[PR];
#pragma unroll
    for (int i = 0; i < PR / 4; ++i) {
        const v4f t = *reinterpret_cast<const v4f*>(rstd + r0 + 4 * i);
        rs[4 * i] = t[0]; rs[4 * i + 1] = t[1]; rs[4 * i + 2] = t[2]; rs[4 * i + 3] = t[3];
    }
    const float s = *d_qscale;
    unsigned wq[PR][2];
#pragma unroll
    for (int i = 0; i < PR; ++i) {
        const v4u o = normalize8(in[i], rs[i], wv);
        if constexpr (WRITE_Y) *reinterpret_cast<v4u*>(y + (r0 + i) * C + c0) = o;
        quantize8<QFMT>(o, s, wq[i][0], wq[i][1]);
    }
    uint8_t* dq = q + r0 * C + c0;
#pragma unroll
    for (int i = 0; i < PR; ++i) {
        v2u v = {wq[i][0], wq[i][1]};
        *reinterpret_cast<v2u*>(dq + (int64_t)i * C) = v;
    }
    if constexpr (TRANSPOSE) {
        uint8_t* dt = qt + c0 * M + r0;
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            unsigned col[4][4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                unsigned blk[4] = {wq[4 * t][k], wq[4 * t + 1][k], wq[4 * t + 2][k], wq[4 * t + 3][k]};
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

// The same for tensors made of whole 128 x 256 tiles: lane geometry and LDS transpose of the quantize kernel's tile
// variant (full 128-byte lines on every stream; the transposed copy optionally in slabs).
template <int QFMT, bool WRITE_Y>
__global__ __launch_bounds__(kTileThreads) void rmsnorm_apply_fp8_tile_kernel(
    const uint16_t* __restrict__ res, const uint16_t* __restrict__ w, const float* __restrict__ rstd,
    int64_t M, int64_t C, const float* __restrict__ d_qscale, uint8_t* __restrict__ q,
    uint8_t* __restrict__ qt, uint16_t* __restrict__ y, unsigned grid_cols, int64_t qt_row_stride,
    int64_t qt_band_stride) {
    __shared__ __attribute__((aligned(16))) uint8_t s_t[kTileLdsBytes];
    const unsigned brow = blockIdx.x / grid_cols, bcol = blockIdx.x - brow * grid_cols;   // along the columns first
    int tr, tc;
    tile_patch_origin(tr, tc);
    const int64_t r0 = (int64_t)brow * kTileRows + tr, c0 = (int64_t)bcol * kTileCols + tc;
    const uint16_t* src = res + r0 * C + c0;
    v4u in[kPatchRows];
#pragma unroll
    for (int i = 0; i < kPatchRows; ++i) in[i] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(src + (int64_t)i * C));
    const v4u wv = *reinterpret_cast<const v4u*>(w + c0);
    float rs[kPatchRows];
#pragma unroll
    for (int i = 0; i < kPatchRows / 4; ++i) {
        const v4f t = *reinterpret_cast<const v4f*>(rstd + r0 + 4 * i);
        rs[4 * i] = t[0]; rs[4 * i + 1] = t[1]; rs[4 * i + 2] = t[2]; rs[4 * i + 3] = t[3];
    }
    const float s = *d_qscale;
    __builtin_amdgcn_sched_barrier(0);
    unsigned wq[kPatchRows][2];
#pragma unroll
    for (int i = 0; i < kPatchRows; ++i) {
        const v4u o = normalize8(in[i], rs[i], wv);
        if constexpr (WRITE_Y) *reinterpret_cast<v4u*>(y + (r0 + i) * C + c0) = o;
        quantize8<QFMT>(o, s, wq[i][0], wq[i][1]);
    }
    uint8_t* dq = q + r0 * C + c0;
#pragma unroll
    for (int i = 0; i < kPatchRows; ++i) *reinterpret_cast<v2u*>(dq + (int64_t)i * C) = v2u{wq[i][0], wq[i][1]};
    tile_stage_transposed(wq, tr, tc, s_t);
    __syncthreads();
    tile_write_transposed(s_t, qt + (int64_t)bcol * kTileCols * qt_row_stride + (int64_t)brow * qt_band_stride, qt_row_stride);
}

template <int QFMT>
__global__ __launch_bounds__(kRnThreads) void rmsnorm_apply_fp8_generic_kernel(
    const uint16_t* __restrict__ res, const uint16_t* __restrict__ w, const float* __restrict__ rstd,
    int64_t M, int64_t C, const float* __restrict__ d_qscale, uint8_t* __restrict__ q,
    uint8_t* __restrict__ qt, uint16_t* __restrict__ y) {
    const int64_t n = M * C;
    const float s = *d_qscale;
    for (int64_t idx = (int64_t)blockIdx.x * kRnThreads + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * kRnThreads) {
        const int64_t m = idx / C, c = idx - m * C;
        const float t = __uint_as_float((unsigned)res[idx] << 16) * rstd[m];
        const unsigned bits = rn_pack(t * __uint_as_float((unsigned)w[c] << 16), 0.0f) & 0xFFFFu;
        if (y) y[idx] = (uint16_t)bits;
        const float p = __uint_as_float(bits << 16) * s;
        const unsigned code = cvt_pair<QFMT>(p, p, 0u, false) & 0xFFu;
        q[idx] = (uint8_t)code;
        if (qt) qt[c * M + m] = (uint8_t)code;
    }
}

int64_t rmsnorm_blocks(int64_t M) { return (M + kRnRowsPerBlock - 1) / kRnRowsPerBlock; }

int launch_rmsnorm_fwd(const void* res_, const void* x_, const void* w_, int64_t M, int64_t C, float eps,
                       void* res_out_, void* y_, float* rstd, unsigned* partial, int fmt, float* d_amax,
                       float* d_scale, hipStream_t stream) {
    const uint16_t* res = reinterpret_cast<const uint16_t*>(res_);
    const uint16_t* x = reinterpret_cast<const uint16_t*>(x_);
    const uint16_t* w = reinterpret_cast<const uint16_t*>(w_);
    uint16_t* res_out = reinterpret_cast<uint16_t*>(res_out_);
    uint16_t* y = reinterpret_cast<uint16_t*>(y_);
    const dim3 grid((unsigned)rmsnorm_blocks(M)), block(kRnThreads);
    if (C % 8 == 0 && C <= kRnMaxC) {
        if (x) hipLaunchKernelGGL((rmsnorm_row_kernel<true>), grid, block, 0, stream, res, x, w, M, (int)C, eps, res_out, y, rstd, partial);
        else hipLaunchKernelGGL((rmsnorm_row_kernel<false>), grid, block, 0, stream, res, x, w, M, (int)C, eps, res_out, y, rstd, partial);
    } else {
        hipLaunchKernelGGL(rmsnorm_row_generic_kernel, grid, block, 0, stream, res, x, w, M, C, eps, res_out, y, rstd, partial);
    }
    if (hipGetLastError() != hipSuccess) return -6;
    return launch_amax_final(partial, (int)rmsnorm_blocks(M), fmt, d_amax, d_scale, stream);
}

static bool use_tile_kernel() {       // LLMQ_FUSED_TILE=0 (tuning override): patch kernels also for whole tiles
    if (const char* e = tuning_env("LLMQ_FUSED_TILE")) return atoi(e) != 0;
    return true;
}

template <int QFMT>
static void launch_apply(const uint16_t* res, const uint16_t* w, const float* rstd, int64_t M, int64_t C,
                         const float* d_qscale, uint8_t* q, uint8_t* q_t, uint16_t* y, hipStream_t stream,
                         bool qt_slabs) {
    const dim3 block(kRnThreads);
    const unsigned gc = (unsigned)((C + kRnBlockCols - 1) / kRnBlockCols);
    if (q_t && tile_shape_ok(M, C) && (qt_slabs || use_tile_kernel())) {
        const unsigned tr = (unsigned)(M / kTileRows), tcn = (unsigned)(C / kTileCols);
        const int64_t row_stride = qt_slabs ? kTileRows : M, band_stride = qt_slabs ? C * kTileRows : kTileRows;
        if (y) hipLaunchKernelGGL((rmsnorm_apply_fp8_tile_kernel<QFMT, true>), dim3(tr * tcn), dim3(kTileThreads), 0, stream, res, w, rstd, M, C, d_qscale, q, q_t, y, tcn, row_stride, band_stride);
        else hipLaunchKernelGGL((rmsnorm_apply_fp8_tile_kernel<QFMT, false>), dim3(tr * tcn), dim3(kTileThreads), 0, stream, res, w, rstd, M, C, d_qscale, q, q_t, y, tcn, row_stride, band_stride);
    } else if (q_t && M % 16 == 0 && C % 8 == 0) {
        const dim3 grid((unsigned)((M + 16 * kRnLanesR - 1) / (16 * kRnLanesR)) * gc);
        if (y) hipLaunchKernelGGL((rmsnorm_apply_fp8_patch_kernel<16, QFMT, true, true>), grid, block, 0, stream, res, w, rstd, M, C, d_qscale, q, q_t, y, gc);
        else hipLaunchKernelGGL((rmsnorm_apply_fp8_patch_kernel<16, QFMT, true, false>), grid, block, 0, stream, res, w, rstd, M, C, d_qscale, q, q_t, y, gc);
    } else if (!q_t && M % 4 == 0 && C % 8 == 0) {
        const dim3 grid((unsigned)((M + 4 * kRnLanesR - 1) / (4 * kRnLanesR)) * gc);
        if (y) hipLaunchKernelGGL((rmsnorm_apply_fp8_patch_kernel<4, QFMT, false, true>), grid, block, 0, stream, res, w, rstd, M, C, d_qscale, q, q_t, y, gc);
        else hipLaunchKernelGGL((rmsnorm_apply_fp8_patch_kernel<4, QFMT, false, false>), grid, block, 0, stream, res, w, rstd, M, C, d_qscale, q, q_t, y, gc);
    } else {
        int64_t blocks = (M * C + kRnThreads - 1) / kRnThreads;
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL((rmsnorm_apply_fp8_generic_kernel<QFMT>), dim3((unsigned)blocks), block, 0, stream, res, w, rstd, M, C, d_qscale, q, q_t, y);
    }
}

int launch_rmsnorm_apply_fp8(const void* res, const void* w, const float* rstd, int64_t M, int64_t C,
                             const float* d_qscale, int fmt, uint8_t* q, uint8_t* q_t, void* y, hipStream_t stream,
                             bool qt_slabs) {
    const uint16_t* r = reinterpret_cast<const uint16_t*>(res);
    const uint16_t* wp = reinterpret_cast<const uint16_t*>(w);
    if (qt_slabs && !(q_t && tile_shape_ok(M, C))) return -2;
    if (fmt == 0) launch_apply<0>(r, wp, rstd, M, C, d_qscale, q, q_t, reinterpret_cast<uint16_t*>(y), stream, qt_slabs);
    else launch_apply<1>(r, wp, rstd, M, C, d_qscale, q, q_t, reinterpret_cast<uint16_t*>(y), stream, qt_slabs);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace llmq
