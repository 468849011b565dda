// FP8 contraction with both operands contraction-contiguous ("TN"), its BF16 baseline, and the kernels for
// shapes no tuned tile divides.  The tile kernel itself is in gemm_tile.h.
#include "gemm_tile.h"

namespace llmq {

void launch_gemm_generic(const uint8_t* A, int fmtA, int layout_a, const uint8_t* B, int fmtB, int layout_b, int64_t R, int64_t C,
                         int64_t T, const float* sA, const float* sB, void* c, int accumulate, unsigned* amax,
                         hipStream_t stream);

// ---- generic kernel: one wavefront per 16x16 outputs, v_mfma_f32_16x16x128_f8f6f4, guarded loads.
// ta / tb: the operand's OperandLayout; the bytes of a T-major operand ([T, R] or [T, Cn]) are gathered one by one.
template <int FA, int FB>
__global__ __launch_bounds__(256) void gemm_generic_kernel(
    const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, uint16_t* __restrict__ C,
    int64_t R, int64_t Cn, int64_t T, const float* __restrict__ d_sA, const float* __restrict__ d_sB,
    int accumulate, unsigned* __restrict__ amax_bits, int ta, int tb) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t r0 = ((int64_t)blockIdx.y * 2 + (wave >> 1)) * 16;
    const int64_t c0 = ((int64_t)blockIdx.x * 2 + (wave & 1)) * 16;
    const int64_t ar = r0 + (lane & 15), bc = c0 + (lane & 15);
    const bool a_ok = ar < R, b_ok = bc < Cn;
    const bool vec_ok = (T % 16) == 0;
    auto load32 = [&](const uint8_t* base, bool ok, int64_t row, int64_t k, int tmajor, int64_t ld) -> v8i {
        v8i v = {0, 0, 0, 0, 0, 0, 0, 0};
        if (!ok || k >= T) return v;
        if (tmajor == kLayoutSlabs) {                 // 32 contiguous bytes of the row's K step (T % 128 == 0)
            const uint8_t* p = base + (k >> 7) * (ld * 128) + row * 128 + (k & 127);
            v4i lo = *reinterpret_cast<const v4i*>(p), hi = *reinterpret_cast<const v4i*>(p + 16);
            return v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
        if (tmajor) {
            for (int w = 0; w < 8; ++w) {
                unsigned word = 0;
                for (int e = 0; e < 4; ++e) {
                    int64_t kk = k + w * 4 + e;
                    if (kk < T) word |= (unsigned)base[kk * ld + row] << (8 * e);
                }
                v[w] = (int)word;
            }
            return v;
        }
        const uint8_t* p = base + row * T + k;
        if (vec_ok && k + 32 <= T) {
            v4i lo = *reinterpret_cast<const v4i*>(p), hi = *reinterpret_cast<const v4i*>(p + 16);
            return v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
        for (int w = 0; w < 8; ++w) {
            unsigned word = 0;
            for (int e = 0; e < 4; ++e) {
                int64_t kk = k + w * 4 + e;
                if (kk < T) word |= (unsigned)p[w * 4 + e] << (8 * e);   // beyond T: code 0x00 = +0
            }
            v[w] = (int)word;
        }
        return v;
    };
    v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int64_t k0 = 0; k0 < T; k0 += 128) {
        const int64_t k = k0 + (lane >> 4) * 32;
        v8i a = load32(A, a_ok, ar, k, ta, R);
        v8i b = load32(B, b_ok, bc, k, tb, Cn);
        acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b, a, acc, FB, FA, 0, 0, 0, 0);
    }
    // lane holds row r0 + lane % 16, columns c0 + 4 * (lane / 16) + 0..3
    const float inv_a = 1.0f / *d_sA, inv_b = 1.0f / *d_sB;
    unsigned mag = 0;
    const int64_t r = r0 + (lane & 15);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int64_t c = c0 + (lane >> 4) * 4 + e;
        if (r < R && c < Cn) {
            float y = acc[e] * inv_a * inv_b;
            uint16_t* dst = C + r * Cn + c;
            if (accumulate) y += __uint_as_float((unsigned)*dst << 16);
            __bf16 o = (__bf16)y;
            unsigned bits = __builtin_bit_cast(uint16_t, o);
            *dst = (uint16_t)bits;
            bits &= 0x7FFFu;
            mag = mag > bits ? mag : bits;
        }
    }
    if (amax_bits) {
        mag = wave_max_u32(mag);
        if (lane == 0) atomicMax(amax_bits, amax_bits_from_bf16_mag(mag));
    }
}

// BF16 operands, any shape: one output element per lane and trip, binary32 accumulation along t.
__global__ __launch_bounds__(256) void gemm_bf16_generic_kernel(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ B, uint16_t* __restrict__ C,
    int64_t R, int64_t Cn, int64_t T, int accumulate) {
    const int64_t n = R * Cn;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = idx / Cn, c = idx - r * Cn;
        float acc = 0.0f;
        for (int64_t t = 0; t < T; ++t)
            acc = __builtin_fmaf(__uint_as_float((unsigned)A[r * T + t] << 16), __uint_as_float((unsigned)B[c * T + t] << 16), acc);
        if (accumulate) acc += __uint_as_float((unsigned)C[idx] << 16);
        C[idx] = __builtin_bit_cast(uint16_t, (__bf16)acc);
    }
}

__global__ void gemm_amax_reset_kernel(unsigned* amax_bits) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *amax_bits = 0u;
}

// ---- host side: tile choice and launch

// Picks the wave tile NI x NJ (workgroup tile 64 NI x 64 NJ) that finishes soonest under a simple
// model: every CU works through its share of the tiles, a tile costs NI * NJ MFMA blocks per K step
// divided by the measured efficiency of that shape relative to 4 x 4 (smaller tiles read more LDS
// and L2 bytes per MFMA; 2 x 2 tiles fit two workgroups per CU, which hide each other's stalls).
TileChoice choose_tile(int64_t R, int64_t C, int64_t T, int num_cus, size_t scratch_bytes) {
    static const float eff[5][5] = {{0, 0, 0, 0, 0}, {0, 0, 0, 0, 0}, {0, 0, 0.90f, 0.74f, 0.77f},
                                    {0, 0, 0.74f, 0.70f, 0.83f}, {0, 0, 0.77f, 0.83f, 1.00f}};
    TileChoice best{0, 0};
    if (T % BK != 0 || T >= (1ll << 23)) return best;
    // Override for tests and tuning: LLMQ_GEMM_TILE=IxJ forces that wave tile where it divides the problem.
    if (const char* force = tuning_env("LLMQ_GEMM_TILE")) {
        const int ni = force[0] - '0', nj = force[0] && force[1] ? force[2] - '0' : 0;
        if (ni >= 2 && ni <= 4 && nj >= 2 && nj <= 4 && R % (64 * ni) == 0 && C % (64 * nj) == 0) return TileChoice{ni, nj};
    }
    double best_cost = 0;
    for (int ni = 4; ni >= 2; --ni)
        for (int nj = 4; nj >= 2; --nj) {
            if (R % (64 * ni) != 0 || C % (64 * nj) != 0) continue;
            const int64_t tiles = (R / (64 * ni)) * (C / (64 * nj));
            if (tiles >= (1ll << 30)) continue;
            const int per_cu = (ni == 2 && nj == 2) ? 2 : 1;          // workgroups resident per CU
            const int64_t slots = resident_slots(num_cus, ni, nj);
            const int64_t rounds = (tiles + slots - 1) / slots;
            // two resident 2 x 2 workgroups overlap each other's prologue and epilogue, which pays most
            // when the contraction is short
            const double e = per_cu == 2 ? (T <= 3072 ? 0.90 : 0.80) : eff[ni][nj];
            // a ragged last round may be shared out among all CUs (choose_split): the model's gain scales the cost
            const SplitChoice sc = choose_split((int)tiles, (int)(T / BK), (int)slots, ni, nj, scratch_bytes);
            const double cost = (double)rounds * per_cu * ni * nj / e * (sc.cost_us / sc.whole_cost_us);
            if (best.ni == 0 || cost < best_cost * 0.97) { best = {ni, nj}; best_cost = cost; }   // larger tile on near ties
        }
    return best;
}

template <int FA, int FB>
static void launch_one(const uint8_t* A, const uint8_t* B, int64_t R, int64_t C, int64_t T,
                       const float* sA, const float* sB, void* c, int accumulate, unsigned* amax,
                       hipStream_t stream, int num_cus, GemmScratch scratch, bool slabs_a = false, bool slabs_b = false) {
    // (an operand in slabs is addressed with 32-bit offsets from its first tile row, 0x7FFFFF00 being out of range)
    const int64_t lim = 0x7FFFFF00ll - ((int64_t)1 << 24);
    const bool fits = (!slabs_a || (T + 256) * R < lim) && (!slabs_b || (T + 256) * C < lim);
    if (fits && launch_chosen_tile<FA, FB, false, false>(A, B, R, C, T, sA, sB, c, accumulate, amax, stream, num_cus, scratch, slabs_a, slabs_b)) return;
    if constexpr (FA == kFmtBf16) {
        const int64_t n = R * C;
        int64_t blocks = (n + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL(gemm_bf16_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                           reinterpret_cast<const uint16_t*>(A), reinterpret_cast<const uint16_t*>(B),
                           reinterpret_cast<uint16_t*>(c), R, C, T / 2, accumulate);
    } else {
        launch_gemm_generic(A, FA, slabs_a ? kLayoutSlabs : kLayoutRows, B, FB, slabs_b ? kLayoutSlabs : kLayoutRows, R, C, T, sA, sB, c,
                            accumulate, amax, stream);
    }
}

void launch_gemm_generic(const uint8_t* A, int fmtA, int ta, const uint8_t* B, int fmtB, int tb, int64_t R, int64_t C,
                         int64_t T, const float* sA, const float* sB, void* c, int accumulate, unsigned* amax,
                         hipStream_t stream) {
    dim3 grid((unsigned)((C + 31) / 32), (unsigned)((R + 31) / 32));
    uint16_t* out = reinterpret_cast<uint16_t*>(c);
    if (fmtA == 0 && fmtB == 0) hipLaunchKernelGGL((gemm_generic_kernel<0, 0>), grid, dim3(256), 0, stream, A, B, out, R, C, T, sA, sB, accumulate, amax, (int)ta, (int)tb);
    else if (fmtA == 1 && fmtB == 0) hipLaunchKernelGGL((gemm_generic_kernel<1, 0>), grid, dim3(256), 0, stream, A, B, out, R, C, T, sA, sB, accumulate, amax, (int)ta, (int)tb);
    else if (fmtA == 0 && fmtB == 1) hipLaunchKernelGGL((gemm_generic_kernel<0, 1>), grid, dim3(256), 0, stream, A, B, out, R, C, T, sA, sB, accumulate, amax, (int)ta, (int)tb);
    else hipLaunchKernelGGL((gemm_generic_kernel<1, 1>), grid, dim3(256), 0, stream, A, B, out, R, C, T, sA, sB, accumulate, amax, (int)ta, (int)tb);
}

void launch_gemm_amax_reset(unsigned* amax, hipStream_t stream) {
    hipLaunchKernelGGL(gemm_amax_reset_kernel, dim3(1), dim3(64), 0, stream, amax);
}

int launch_gemm_tn(const uint8_t* A, int fmtA, const uint8_t* B, int fmtB, int64_t R, int64_t C,
                   int64_t T, const float* d_scaleA, const float* d_scaleB, void* c_bf16,
                   int accumulate, float* d_amax_c, bool amax_is_zeroed, hipStream_t stream, int num_cus, GemmScratch scratch,
                   bool slabs_a, bool slabs_b) {
    unsigned* amax = reinterpret_cast<unsigned*>(d_amax_c);
    if (amax && !amax_is_zeroed) hipLaunchKernelGGL(gemm_amax_reset_kernel, dim3(1), dim3(64), 0, stream, amax);
    if (fmtA == 0 && fmtB == 0) launch_one<0, 0>(A, B, R, C, T, d_scaleA, d_scaleB, c_bf16, accumulate, amax, stream, num_cus, scratch, slabs_a, slabs_b);
    else if (fmtA == 1 && fmtB == 0) launch_one<1, 0>(A, B, R, C, T, d_scaleA, d_scaleB, c_bf16, accumulate, amax, stream, num_cus, scratch, slabs_a, slabs_b);
    else if (fmtA == 0 && fmtB == 1) launch_one<0, 1>(A, B, R, C, T, d_scaleA, d_scaleB, c_bf16, accumulate, amax, stream, num_cus, scratch, slabs_a, slabs_b);
    else launch_one<1, 1>(A, B, R, C, T, d_scaleA, d_scaleB, c_bf16, accumulate, amax, stream, num_cus, scratch, slabs_a, slabs_b);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

// Scratch a launch of this shape would use when given as much as it likes (0: every tile is computed whole).
size_t gemm_scratch_bytes(int64_t R, int64_t C, int64_t T, int num_cus) {
    const size_t unlimited = ~(size_t)0;
    const TileChoice tc = choose_tile(R, C, T, num_cus, unlimited);
    if (tc.ni == 0) return 0;
    const int64_t tiles = (R / (64 * tc.ni)) * (C / (64 * tc.nj));
    const SplitChoice sc = choose_split((int)tiles, (int)(T / BK), resident_slots(num_cus, tc.ni, tc.nj), tc.ni, tc.nj, unlimited);
    return sc.slots * (size_t)(4 * 4096 * tc.ni * tc.nj);
}

// Phase stamps of the 256 x 256 tile kernel (E4M3 x E4M3, contraction-contiguous operands): the same kernel with
// kProfile, which makes wave 0 of every workgroup record cycle and 100 MHz stamps of its phases, 16 words of 64 bits
// per workgroup id (see GemmTuning::kProfile).
template <bool IEEE>
struct GemmPhaseTuning : GemmTuning {
    static constexpr bool kProfile = true;
    static constexpr bool kIeeeMaximum = IEEE;
    static __device__ void record(float* buf, int block, int slot, long long value) {
        reinterpret_cast<long long*>(buf)[(size_t)block * 16 + slot] = value;
    }
};

int gemm_phase_stamp_blocks(int64_t R, int64_t C) { return (int)((((R / 256) * (C / 256) + kXcds - 1) / kXcds) * kXcds); }

int launch_gemm_phase_stamps(const uint8_t* A, const uint8_t* B, int64_t R, int64_t C, int64_t T, const float* sA,
                             const float* sB, void* c_bf16, float* d_amax_c, long long* stamps, int ieee_maximum,
                             hipStream_t stream, int num_cus) {
    const int tiles_r = (int)(R / 256), tiles_c = (int)(C / 256), nt = tiles_r * tiles_c;
    const int grid = gemm_phase_stamp_blocks(R, C);
    const int slots = resident_slots(num_cus, 4, 4);
    const int band = band_rows();
    const int share_b = band < tiles_r ? band : tiles_r, share_a = 4 < tiles_c ? 4 : tiles_c;
    const int next_stride = touch_next(nt >= 6 * slots) ? slots : 0;
    SplitPlan plan{};
    plan.n_whole = nt;
    plan.partials = reinterpret_cast<float*>(stamps);
    unsigned* amax = reinterpret_cast<unsigned*>(d_amax_c);
    hipLaunchKernelGGL(gemm_amax_reset_kernel, dim3(1), dim3(64), 0, stream, amax);
    auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(kGemmThreads), 0, stream, A, B, reinterpret_cast<uint16_t*>(c_bf16),
                           (int)C, (int)T, sA, sB, amax, tiles_r, tiles_c, touch_ahead(), band, next_stride, (int)T, (int)T,
                           BK, BK, share_a, share_b, plan);
    };
    if (ieee_maximum) launch(gemm_tile_kernel<0, 0, 4, 4, false, GemmPhaseTuning<true>>);
    else launch(gemm_tile_kernel<0, 0, 4, 4, false, GemmPhaseTuning<false>>);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

// BF16 baseline: same tile kernels with the BF16 MFMA; T counts elements here, rows are 2 T bytes long.
int launch_gemm_bf16_tn(const void* A, const void* B, int64_t R, int64_t C, int64_t T, void* c_bf16,
                        int accumulate, hipStream_t stream, int num_cus) {
    launch_one<kFmtBf16, kFmtBf16>(reinterpret_cast<const uint8_t*>(A), reinterpret_cast<const uint8_t*>(B), R, C, 2 * T,
                                   nullptr, nullptr, c_bf16, accumulate, nullptr, stream, num_cus, GemmScratch{nullptr, 0});
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace llmq
