// Fused scale + FP8 cast + transposed copy (paper Section 3, kernel-fusion paragraph: quantization and
// transposition are one kernel; the FP8 GEMM wants both operands contraction-contiguous, so every
// quantized tensor is also needed transposed in the backward pass).
//
// HBM-bound: per element 2 bytes read, 1 byte written row-major and 1 byte written transposed.
// Tuned kernel: one lane owns a 16-row x 8-column patch.  It reads the patch with sixteen 16-byte
// loads (eight lanes side by side cover a full 128-byte line of a row), converts with one binary32
// multiply and the hardware RNE cast (clamped first, which makes it saturating), writes its 8 bytes
// of each row, transposes the 16x8 byte patch in registers with byte permutes and writes eight
// 16-byte vectors of the transposed tensor (eight lanes stacked in rows cover a full 128-byte line
// there).  No LDS, no barrier.
#include <stdlib.h>

#include "llmq_device.h"
#include "llmq_kernels.h"

namespace llmq {

constexpr int kQThreads = 256;

// Shape of the work of one wavefront: every lane owns a patch of 16 rows x kPatchCols columns,
// kLanesR lanes are stacked along rows (16 * kLanesR rows per wave, which is also the length in
// bytes of the contiguous pieces written to the transposed tensor) and 64 / kLanesR lanes sit side
// by side along columns.  The four waves of a workgroup sit side by side along columns.
struct QuantTuning {
    static constexpr int kPatchCols = 8;     // 8 or 16 (one or two 16-byte loads per row)
    static constexpr int kLanesR = 8;
    static constexpr bool kLoadsFirst = true;    // issue every load of the patch before the first conversion
    static constexpr bool kNtLoad = true;        // streaming hint on the loads
    static constexpr bool kNtStore = false;      // streaming hint on the stores
    // Block columns per band of the workgroup walk (see the kernel).  Measured on the benchmark tensors:
    // walking along the columns (one band) beats walking down the rows (band = 1) by 1-4 %, bands of 2-16 lie
    // in between.  LLMQ_QUANT_BAND overrides it for tuning.
    static constexpr int kBandBlocks = 1 << 20;
};

template <int FMT, bool TRANSPOSE, class V = QuantTuning>
__global__ __launch_bounds__(kQThreads) void quantize_patch_kernel(
    const uint16_t* __restrict__ x, int64_t rows, int64_t cols, const ScaleSource scale_src,
    uint8_t* __restrict__ q, uint8_t* __restrict__ qt, unsigned* __restrict__ zero_word,
    unsigned grid_rows, unsigned grid_cols, unsigned band) {
    __shared__ unsigned s_part[kQThreads / kWave];
    if (zero_word && blockIdx.x == 0 && threadIdx.x == 0) *zero_word = 0u;
    const float s = resolve_scale(scale_src, blockIdx.x == 0, s_part);   // before any lane leaves
    // Workgroup id -> block of the tensor: bands of `band` block columns, walked down the rows, `band`
    // neighbouring blocks of a row one after the other.  Workgroups in flight together then read runs of
    // band * 512 bytes of a row and write runs of the transposed tensor's rows that keep growing as the walk
    // moves down (band = 1: plain walk down the rows; band >= grid_cols: along the columns).
    unsigned brow, bcol;
    band_walk(blockIdx.x, grid_rows, grid_cols, band, brow, bcol);
    constexpr int PC = V::kPatchCols, LR = V::kLanesR, LC = kWave / LR;
    constexpr int NV = PC / 8;                              // 16-byte loads per row of the patch
    constexpr int kWaveRows = kPatchRows * LR, kWaveCols = PC * LC;
    constexpr int kBlockCols = kWaveCols * (kQThreads / kWave);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t r0 = (int64_t)brow * kWaveRows + (lane % LR) * kPatchRows;
    const int64_t c0 = (int64_t)bcol * kBlockCols + wave * kWaveCols + (lane / LR) * PC;
    if (r0 >= rows || c0 >= cols) return;       // rows % 16 == 0 and cols % PC == 0: a patch is all in or all out
    v4u in[kPatchRows][NV];
    const uint16_t* src = x + r0 * cols + c0;
#pragma unroll
    for (int i = 0; i < kPatchRows; ++i)
#pragma unroll
        for (int v = 0; v < NV; ++v)
            in[i][v] = V::kNtLoad ? __builtin_nontemporal_load(reinterpret_cast<const v4u*>(src + (int64_t)i * cols) + v)
                                       : *(reinterpret_cast<const v4u*>(src + (int64_t)i * cols) + v);
    if constexpr (V::kLoadsFirst) __builtin_amdgcn_sched_barrier(0);
    unsigned w[kPatchRows][2 * NV];             // the patch as FP8 bytes: w[row][k] = columns 4k .. 4k+3
#pragma unroll
    for (int i = 0; i < kPatchRows; ++i)
#pragma unroll
        for (int v = 0; v < NV; ++v) quantize8<FMT>(in[i][v], s, w[i][2 * v], w[i][2 * v + 1]);
    uint8_t* dst = q + r0 * cols + c0;
#pragma unroll
    for (int i = 0; i < kPatchRows; ++i) {
        if constexpr (NV == 1) {
            v2u v = {w[i][0], w[i][1]};
            if constexpr (V::kNtStore) __builtin_nontemporal_store(v, reinterpret_cast<v2u*>(dst + (int64_t)i * cols));
            else *reinterpret_cast<v2u*>(dst + (int64_t)i * cols) = v;
        } else {
            v4u v = {w[i][0], w[i][1], w[i][2], w[i][3]};
            if constexpr (V::kNtStore) __builtin_nontemporal_store(v, reinterpret_cast<v4u*>(dst + (int64_t)i * cols));
            else *reinterpret_cast<v4u*>(dst + (int64_t)i * cols) = v;
        }
    }
    if constexpr (TRANSPOSE) {
        // column j of the patch -> 16 consecutive bytes of row (c0 + j) of the transposed tensor
        uint8_t* dt = qt + c0 * rows + r0;
#pragma unroll
        for (int k = 0; k < 2 * NV; ++k) {      // four columns at a time
            unsigned col[4][4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {       // four rows at a time
                unsigned blk[4] = {w[4 * t][k], w[4 * t + 1][k], w[4 * t + 2][k], w[4 * t + 3][k]};
                unsigned o[4];
                transpose4x4_bytes(blk, o);
#pragma unroll
                for (int c = 0; c < 4; ++c) col[c][t] = o[c];
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                v4u v = {col[c][0], col[c][1], col[c][2], col[c][3]};
                if constexpr (V::kNtStore) __builtin_nontemporal_store(v, reinterpret_cast<v4u*>(dt + (int64_t)(4 * k + c) * rows));
                else *reinterpret_cast<v4u*>(dt + (int64_t)(4 * k + c) * rows) = v;
            }
        }
    }
}

// Workgroup-tile variant for tensors whose rows are a multiple of 128 and whose columns a multiple of 256 (every
// benchmark tensor): full 128-byte lines on all three streams.  A lane owns the same 16 x 8 patch, but a wave is
// 4 lanes stacked x 16 side by side, and the transposed copy cannot be written that way from registers (4 stacked
// lanes hold 64 contiguous bytes of a transposed row), so the transposed patches go through LDS (the tile_*
// helpers).
template <int FMT>
__global__ __launch_bounds__(kTileThreads) void quantize_tile_kernel(
    const uint16_t* __restrict__ x, int64_t rows, int64_t cols, const ScaleSource scale_src,
    uint8_t* __restrict__ q, uint8_t* __restrict__ qt, unsigned* __restrict__ zero_word, unsigned grid_cols,
    int64_t qt_row_stride, int64_t qt_band_stride) {
    __shared__ unsigned s_part[kTileThreads / kWave];
    __shared__ __attribute__((aligned(16))) uint8_t s_t[kTileLdsBytes];
    if (zero_word && blockIdx.x == 0 && threadIdx.x == 0) *zero_word = 0u;
    const float s = resolve_scale(scale_src, blockIdx.x == 0, s_part);
    const unsigned brow = blockIdx.x / grid_cols, bcol = blockIdx.x - brow * grid_cols;   // along the columns first
    int tr, tc;
    tile_patch_origin(tr, tc);
    const int64_t r0 = (int64_t)brow * kTileRows + tr, c0 = (int64_t)bcol * kTileCols + tc;
    v4u in[kPatchRows];
    const uint16_t* src = x + r0 * cols + c0;
#pragma unroll
    for (int i = 0; i < kPatchRows; ++i) in[i] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(src + (int64_t)i * cols));
    __builtin_amdgcn_sched_barrier(0);
    unsigned w[kPatchRows][2];
#pragma unroll
    for (int i = 0; i < kPatchRows; ++i) quantize8<FMT>(in[i], s, w[i][0], w[i][1]);
    uint8_t* dst = q + r0 * cols + c0;
#pragma unroll
    for (int i = 0; i < kPatchRows; ++i) *reinterpret_cast<v2u*>(dst + (int64_t)i * cols) = v2u{w[i][0], w[i][1]};
    tile_stage_transposed(w, tr, tc, s_t);
    __syncthreads();
    // (qt_row_stride, qt_band_stride) = (rows, 128) for the transposed tensor as such, (128, cols x 128) in slabs
    tile_write_transposed(s_t, qt + (int64_t)bcol * kTileCols * qt_row_stride + (int64_t)brow * qt_band_stride, qt_row_stride);
}

// No transposed copy wanted: the conversion is element-wise and the tensor can be taken as a flat array.  A
// workgroup converts kFlatUnits * 256 runs of 8 elements; load j of a wave covers 1 KB of contiguous input,
// its store 512 contiguous bytes (the patch kernel without the transposed copy writes 64-byte pieces of rows and
// reaches 4.8-5.2 TB/s where this one reaches 5.9-6.1; with 1, 4 or 8 runs per lane instead of 2: 2-7 % less).
constexpr int kFlatUnits = 2;

template <int FMT>
__global__ __launch_bounds__(kQThreads) void quantize_flat_kernel(
    const uint16_t* __restrict__ x, int64_t n8, const ScaleSource scale_src, uint8_t* __restrict__ q,
    unsigned* __restrict__ zero_word) {
    __shared__ unsigned s_part[kQThreads / kWave];
    if (zero_word && blockIdx.x == 0 && threadIdx.x == 0) *zero_word = 0u;
    const float s = resolve_scale(scale_src, blockIdx.x == 0, s_part);
    const int64_t first = (int64_t)blockIdx.x * (kQThreads * kFlatUnits) + threadIdx.x;
    v4u in[kFlatUnits];
#pragma unroll
    for (int j = 0; j < kFlatUnits; ++j) {
        const int64_t u = first + j * kQThreads;
        if (u < n8) in[j] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(x) + u);
    }
#pragma unroll
    for (int j = 0; j < kFlatUnits; ++j) {
        const int64_t u = first + j * kQThreads;
        if (u < n8) {
            unsigned lo, hi;
            quantize8<FMT>(in[j], s, lo, hi);
            *(reinterpret_cast<v2u*>(q) + u) = v2u{lo, hi};
        }
    }
}

// Any shape: one element per lane.  Lanes run along columns for the read and the row-major write.
template <int FMT>
__global__ __launch_bounds__(256) void quantize_generic_kernel(
    const uint16_t* __restrict__ x, int64_t rows, int64_t cols, const ScaleSource scale_src,
    uint8_t* __restrict__ q, uint8_t* __restrict__ qt, unsigned* __restrict__ zero_word) {
    __shared__ unsigned s_part[256 / kWave];
    if (zero_word && blockIdx.x == 0 && threadIdx.x == 0) *zero_word = 0u;
    const int64_t n = rows * cols;
    const float s = resolve_scale(scale_src, blockIdx.x == 0, s_part);
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        float p = __uint_as_float((unsigned)x[i] << 16) * s;
        unsigned code = cvt_pair<FMT>(p, p, 0u, false) & 0xFFu;
        q[i] = (uint8_t)code;
        if (qt) {
            int64_t r = i / cols, c = i - r * cols;
            qt[c * rows + r] = (uint8_t)code;
        }
    }
}

template <class V>
static void launch_patch(const uint16_t* xb, int64_t rows, int64_t cols, const ScaleSource& d_scale, int fmt,
                         uint8_t* q, uint8_t* q_t, unsigned* zero_word, hipStream_t stream) {
    constexpr int kWaveRows = kPatchRows * V::kLanesR;
    constexpr int kBlockCols = V::kPatchCols * (kWave / V::kLanesR) * (kQThreads / kWave);
    const unsigned gc = (unsigned)((cols + kBlockCols - 1) / kBlockCols), gr = (unsigned)((rows + kWaveRows - 1) / kWaveRows);
    dim3 grid(gr * gc);
    dim3 block(kQThreads);
    unsigned band = V::kBandBlocks;
    if (const char* e = tuning_env("LLMQ_QUANT_BAND")) { const int v = atoi(e); if (v >= 1) band = (unsigned)v; }
    if (band > gc) band = gc;      // band * gr then stays within the grid size, which fits 32 bits
    if (fmt == 0) {
        if (q_t) hipLaunchKernelGGL((quantize_patch_kernel<0, true, V>), grid, block, 0, stream, xb, rows, cols, d_scale, q, q_t, zero_word, gr, gc, band);
        else hipLaunchKernelGGL((quantize_patch_kernel<0, false, V>), grid, block, 0, stream, xb, rows, cols, d_scale, q, q_t, zero_word, gr, gc, band);
    } else {
        if (q_t) hipLaunchKernelGGL((quantize_patch_kernel<1, true, V>), grid, block, 0, stream, xb, rows, cols, d_scale, q, q_t, zero_word, gr, gc, band);
        else hipLaunchKernelGGL((quantize_patch_kernel<1, false, V>), grid, block, 0, stream, xb, rows, cols, d_scale, q, q_t, zero_word, gr, gc, band);
    }
}

// LLMQ_QUANT_TILE=0 / 1 (tuning override): the register-only patch kernel or the workgroup-tile kernel.
static bool use_tile_kernel() {
    if (const char* e = tuning_env("LLMQ_QUANT_TILE")) return atoi(e) != 0;
    return true;
}

int launch_quantize(const void* x, int64_t rows, int64_t cols, const float* d_scale, int fmt,
                    uint8_t* q, uint8_t* q_t, unsigned* zero_word, hipStream_t stream, bool qt_slabs) {
    const ScaleSource src{d_scale, nullptr, 0, fp8_max(fmt), nullptr};
    return launch_quantize_from(x, rows, cols, src, fmt, q, q_t, zero_word, stream, qt_slabs);
}

bool quantize_can_write_slabs(int64_t rows, int64_t cols) {
    return tile_shape_ok(rows, cols) && use_tile_kernel();
}

int launch_quantize_from(const void* x, int64_t rows, int64_t cols, const ScaleSource& d_scale, int fmt,
                         uint8_t* q, uint8_t* q_t, unsigned* zero_word, hipStream_t stream, bool qt_slabs) {
    const uint16_t* xb = reinterpret_cast<const uint16_t*>(x);
    if (qt_slabs && !(q_t && quantize_can_write_slabs(rows, cols))) return -2;       // the caller asks first
    if (!q_t && (rows * cols) % 8 == 0) {
        const int64_t n8 = rows * cols / 8;
        const dim3 grid((unsigned)((n8 + kQThreads * kFlatUnits - 1) / (kQThreads * kFlatUnits)));
        if (fmt == 0) hipLaunchKernelGGL((quantize_flat_kernel<0>), grid, dim3(kQThreads), 0, stream, xb, n8, d_scale, q, zero_word);
        else hipLaunchKernelGGL((quantize_flat_kernel<1>), grid, dim3(kQThreads), 0, stream, xb, n8, d_scale, q, zero_word);
    } else if (q_t && tile_shape_ok(rows, cols) && use_tile_kernel()) {
        const unsigned gc = (unsigned)(cols / kTileCols), gr = (unsigned)(rows / kTileRows);
        const int64_t row_stride = qt_slabs ? kTileRows : rows, band_stride = qt_slabs ? cols * kTileRows : kTileRows;
        if (fmt == 0) hipLaunchKernelGGL((quantize_tile_kernel<0>), dim3(gr * gc), dim3(kQThreads), 0, stream, xb, rows, cols, d_scale, q, q_t, zero_word, gc, row_stride, band_stride);
        else hipLaunchKernelGGL((quantize_tile_kernel<1>), dim3(gr * gc), dim3(kQThreads), 0, stream, xb, rows, cols, d_scale, q, q_t, zero_word, gc, row_stride, band_stride);
    } else if (rows % kPatchRows == 0 && cols % QuantTuning::kPatchCols == 0) {
        launch_patch<QuantTuning>(xb, rows, cols, d_scale, fmt, q, q_t, zero_word, stream);
    } else {
        int64_t n = rows * cols;
        int64_t blocks = (n + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        if (fmt == 0) hipLaunchKernelGGL((quantize_generic_kernel<0>), dim3((unsigned)blocks), dim3(256), 0, stream, xb, rows, cols, d_scale, q, q_t, zero_word);
        else hipLaunchKernelGGL((quantize_generic_kernel<1>), dim3((unsigned)blocks), dim3(256), 0, stream, xb, rows, cols, d_scale, q, q_t, zero_word);
    }
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace llmq
