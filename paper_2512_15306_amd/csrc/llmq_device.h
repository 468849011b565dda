// Device-side helpers shared by the gfx950 kernels of the FP8 linear path.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "llmq_kernels.h"

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

// Packed maximum of the magnitudes (bits & 0x7FFF) of the two BF16 values in w with the pair in acc.
__device__ inline unsigned pk_max_mag(unsigned acc, unsigned w) {
    v2us a = __builtin_bit_cast(v2us, acc);
    v2us b = __builtin_bit_cast(v2us, w & 0x7FFF7FFFu);
    return __builtin_bit_cast(unsigned, __builtin_elementwise_max(a, b));
}

// Maximum over a workgroup of THREADS lanes; s_part holds one word per wavefront.
template <int THREADS>
__device__ inline unsigned block_max_u32(unsigned m, unsigned* s_part) {
    m = wave_max_u32(m);
    if ((threadIdx.x & (kWave - 1)) == 0) s_part[threadIdx.x / kWave] = m;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < THREADS / kWave; ++w) m = m > s_part[w] ? m : s_part[w];
    return m;
}

// The scale of a tensor whose absmax is a (paper Section 3 "Overview": the absmax is mapped onto the largest
// finite FP8 value): fmax / a with one correctly rounded binary32 division, FLT_MAX when that quotient
// overflows (a tiny absmax), and 1 for an all-zero tensor, where the rule defines nothing and every scale
// gives the same codes (+-0): the neutral scale keeps the de-scaling exact and stays usable as a kept statistic.
// a = +Inf gives 0, a = NaN gives NaN.
__device__ inline float scale_of_amax(float a, float fmax) {
    float s = fmax / a;
    if (__builtin_isinf(s)) s = a == 0.0f ? 1.0f : 3.402823466e+38f;
    return s;
}

// The same from a BF16 magnitude pattern, as the absmax second stage computes it
__device__ inline float scale_from_mag(unsigned mag16, float fmax) {
    return scale_of_amax(__uint_as_float(amax_bits_from_bf16_mag(mag16)), fmax);
}

// The scale of a 256-lane workgroup's launch; all lanes of the workgroup must call it.
__device__ inline float resolve_scale(const ScaleSource& src, bool first_block, unsigned* s_part) {
    if (src.partial == nullptr) return *src.d_scale;
    unsigned m = 0;
    for (int i = threadIdx.x; i < src.n_partial; i += 256) {
        const unsigned v = src.partial[i];
        m = m > v ? m : v;
    }
    m = block_max_u32<256>(m, s_part);
    const float s = scale_from_mag(m, src.fmax);
    if (first_block && threadIdx.x == 0) *src.d_scale_out = s;
    return s;
}

// Workgroup id -> block (brow, bcol) of a grid of grid_rows x grid_cols blocks: bands of `band` block columns
// (1 <= band <= grid_cols, so that band * grid_rows stays within the grid size, which fits 32 bits), walked down
// the rows, `band` neighbouring blocks of a row one after the other; the last band takes the columns that are
// left.  band = 1: down the rows; band = grid_cols: along the columns.
__host__ __device__ inline void band_walk(unsigned id, unsigned grid_rows, unsigned grid_cols, unsigned band,
                                          unsigned& brow, unsigned& bcol) {
    const unsigned band_first = (id / (band * grid_rows)) * band;
    const unsigned band_width = grid_cols - band_first < band ? grid_cols - band_first : band;
    const unsigned in_band = id - band_first * grid_rows;
    brow = in_band / band_width;
    bcol = band_first + in_band % band_width;
}

// ---- FP8 cast helpers (used by the quantize kernel and by the producers that emit FP8 directly) ----

template <int FMT>
__device__ inline unsigned cvt_pair(float a, float b, unsigned old, bool high) {
    constexpr float fmax = FMT == 0 ? 448.0f : 57344.0f;
    a = __builtin_amdgcn_fmed3f(a, -fmax, fmax);         // saturate; the cast below rounds to nearest even
    b = __builtin_amdgcn_fmed3f(b, -fmax, fmax);
    if constexpr (FMT == 0) {
        return high ? (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, (int)old, true)
                    : (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, (int)old, false);
    } else {
        return high ? (unsigned)__builtin_amdgcn_cvt_pk_bf8_f32(a, b, (int)old, true)
                    : (unsigned)__builtin_amdgcn_cvt_pk_bf8_f32(a, b, (int)old, false);
    }
}

// Four BF16 pairs (one 16-byte load) -> eight FP8 codes in two dwords.
template <int FMT>
__device__ inline void quantize8(const v4u& r, float s, unsigned& lo, unsigned& hi) {
    float f[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f[2 * j] = __uint_as_float(r[j] << 16) * s;            // even element: low half of the dword
        f[2 * j + 1] = __uint_as_float(r[j] & 0xFFFF0000u) * s;
    }
    lo = cvt_pair<FMT>(f[0], f[1], 0u, false);
    lo = cvt_pair<FMT>(f[2], f[3], lo, true);
    hi = cvt_pair<FMT>(f[4], f[5], 0u, false);
    hi = cvt_pair<FMT>(f[6], f[7], hi, true);
}

// w[r] holds bytes (r,0..3) of a 4x4 byte block; returns o[c] = bytes (0..3,c).
__device__ inline void transpose4x4_bytes(const unsigned w[4], unsigned o[4]) {
    // v_perm_b32 selects from the 8 bytes {first operand: 4..7, second operand: 0..3}
    unsigned t01l = __builtin_amdgcn_perm(w[1], w[0], 0x05010400u);   // w0.0 w1.0 w0.1 w1.1
    unsigned t01h = __builtin_amdgcn_perm(w[1], w[0], 0x07030602u);   // w0.2 w1.2 w0.3 w1.3
    unsigned t23l = __builtin_amdgcn_perm(w[3], w[2], 0x05010400u);
    unsigned t23h = __builtin_amdgcn_perm(w[3], w[2], 0x07030602u);
    o[0] = __builtin_amdgcn_perm(t23l, t01l, 0x05040100u);
    o[1] = __builtin_amdgcn_perm(t23l, t01l, 0x07060302u);
    o[2] = __builtin_amdgcn_perm(t23h, t01h, 0x05040100u);
    o[3] = __builtin_amdgcn_perm(t23h, t01h, 0x07060302u);
}

// ---- The 128-row x 256-column workgroup tile of the kernels that write FP8 codes in both layouts ----
//
// 256 lanes; a lane owns a patch of 16 rows x 8 columns, a wave is 4 lanes stacked x 16 side by side (64 rows x 128
// columns: its loads of BF16 input cover 256 contiguous bytes of a row, its stores of codes a whole 128-byte line),
// the four waves tile 128 x 256.  The transposed patches (16-byte column pieces after the register transpose)
// go through a [256 columns][128 rows] byte tile in LDS (rows padded to 144 bytes against bank conflicts) and
// leave, after one barrier, as 128-byte lines of the transposed tensor, 8 lanes per transposed row.
constexpr int kTilePitch = kTileRows + 16;        // kTileRows = 128, kTileCols = 256
constexpr int kTileThreads = 256, kPatchRows = 16;
constexpr int kTileLdsBytes = kTileCols * kTilePitch;

// Origin of this lane's patch inside the tile
__device__ inline void tile_patch_origin(int& tr, int& tc) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    tr = (wave >> 1) * 64 + (lane & 3) * kPatchRows;
    tc = (wave & 1) * 128 + (lane >> 2) * 8;
}

// The patch as FP8 bytes, w[row][k] = columns 4k .. 4k+3: column j of the patch becomes 16 consecutive bytes of
// row (tc + j) of the LDS tile, at byte tr.
__device__ inline void tile_stage_transposed(const unsigned (&w)[kPatchRows][2], int tr, int tc, uint8_t* s_t) {
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        unsigned col[4][4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            unsigned blk[4] = {w[4 * t][k], w[4 * t + 1][k], w[4 * t + 2][k], w[4 * t + 3][k]};
            unsigned o[4];
            transpose4x4_bytes(blk, o);
#pragma unroll
            for (int c = 0; c < 4; ++c) col[c][t] = o[c];
        }
#pragma unroll
        for (int c = 0; c < 4; ++c)
            *reinterpret_cast<v4u*>(s_t + (tc + 4 * k + c) * kTilePitch + tr) = v4u{col[c][0], col[c][1], col[c][2], col[c][3]};
    }
}

// After the barrier that follows the staging: the whole tile to memory.  dt = where transposed row 0 of this tile
// starts; transposed row c starts row_stride bytes after row c - 1.  The transposed tensor [cols, rows] as such:
// dt = qt + (first column) rows + (first row), row_stride = rows.  In slabs of 128 contraction bytes
// (OperandLayout): dt = qt + (first row / 128) cols 128 + (first column) 128, row_stride = 128, and the tile's
// 32 KB are one contiguous piece.
__device__ inline void tile_write_transposed(const uint8_t* s_t, uint8_t* dt, int64_t row_stride) {
#pragma unroll
    for (int m = 0; m < kTileCols * (kTileRows / 16) / kTileThreads; ++m) {
        const int p = threadIdx.x + m * kTileThreads;       // 16-byte piece: column p / 8, rows 16 (p % 8) ..
        const int c = p >> 3, ch = p & 7;
        const v4u v = *reinterpret_cast<const v4u*>(s_t + c * kTilePitch + ch * 16);
        *reinterpret_cast<v4u*>(dt + (int64_t)c * row_stride + ch * 16) = v;
    }
}

}  // namespace llmq
