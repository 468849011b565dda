// FP8 contraction on the gfx950 matrix cores (paper Section 3: the transformer-block matmuls of
// forward and backward run in FP8, results stay in BF16; the FP8 GEMM is "TN", i.e. both operands
// have the contraction index contiguous).
//
//   C[r,c] = bf16( (sum_t A[r,t] * B[c,t]) / (sA * sB) ),   A [R,T] fp8, B [Cn,T] fp8.
//
// Tuned kernel (R, Cn multiples of 256; T a multiple of 128)
//   - one workgroup of 4 wavefronts per 256x256 output tile, each wavefront owns 128x128 of it
//     as 4x4 blocks of v_mfma_f32_32x32x64_f8f6f4 (fp32 accumulators, 256 registers per lane);
//   - K advances 128 bytes per step; the A and B slabs (256 rows x 128 B each) go from global memory
//     straight into LDS with buffer_load ... lds (16 bytes per lane, no VGPR staging), double
//     buffered: 2 x 64 KB of the 160 KB LDS;
//   - LDS rows are 128 B; the 16-byte chunk index is XOR-ed with (row & 7), applied on the global
//     side of the load, so that the ds_read_b128 fragment reads of 8 consecutive rows hit all banks;
//   - the order of the contraction index inside one MFMA does not matter as long as A and B use
//     the same order, so every lane simply reads 32 contiguous bytes of its row;
//   - the MFMA takes the B rows as its first operand, which leaves every lane with 4 consecutive
//     output columns of one row: the epilogue de-scales in fp32, rounds to BF16 with the hardware
//     conversion and stores 8 bytes per lane; the output absmax is taken on the rounded BF16 bits;
//   - workgroup ids are dealt round-robin to the 8 XCDs by the hardware, so ids are remapped to give
//     each XCD (own L2) a contiguous range of tiles, walked in bands 8 tile-rows high.
// Generic kernel: any shape, one wavefront per 16x16 outputs, guarded loads; slow, for tests and
// odd sizes.
#include "llmq_device.h"
#include "llmq_kernels.h"

namespace llmq {

typedef __attribute__((address_space(3))) void lds_void;
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 256, BN = 256, BK = 128;
constexpr int kGemmThreads = 256;
constexpr int kSlabBytes = BM * BK;                 // 32 KB per operand per stage
constexpr int kXcds = 8;
constexpr int kBandRows = 8;

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
    // raw buffer, no stride; out-of-range reads return zero instead of faulting
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

__device__ inline unsigned bf16_mag_max4(unsigned m, bf16x4 v) {
    v2u w = __builtin_bit_cast(v2u, v);
    unsigned a = w[0] & 0x7FFF7FFFu, b = w[1] & 0x7FFF7FFFu;
    unsigned x = (a & 0xFFFFu) > (a >> 16) ? (a & 0xFFFFu) : (a >> 16);
    unsigned y = (b & 0xFFFFu) > (b >> 16) ? (b & 0xFFFFu) : (b >> 16);
    x = x > y ? x : y;
    return m > x ? m : x;
}

// Linear workgroup id -> output tile, XCD-aware.  Returns false for the padding ids.
__device__ inline bool tile_of_block(int pid, int tiles_r, int tiles_c, int& tr, int& tc) {
    const int nt = tiles_r * tiles_c;
    const int per_xcd = (nt + kXcds - 1) / kXcds;
    const int id = (pid % kXcds) * per_xcd + pid / kXcds;
    if (id >= nt) return false;
    const int band = kBandRows * tiles_c;
    const int first = (id / band) * kBandRows;
    const int h = tiles_r - first < kBandRows ? tiles_r - first : kBandRows;
    const int in_band = id % band;
    tr = first + in_band % h;
    tc = in_band / h;
    return true;
}

// MFMA scheduling masks of __builtin_amdgcn_sched_group_barrier
constexpr int kSchedMfma = 0x008, kSchedVmemRead = 0x020, kSchedDsRead = 0x100;

template <int FA, int FB>
__device__ inline void mma_4x4(v16f (&acc)[4][4], const v8i (&a)[4], const v8i (&b)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b[j], a[i], acc[i][j], FB, FA, 0, 0, 0, 0);
}

template <int FA, int FB>
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_tn_256_kernel(
    const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, uint16_t* __restrict__ C,
    int Cn, int T, const float* __restrict__ d_sA, const float* __restrict__ d_sB,
    int accumulate, unsigned* __restrict__ amax_bits, int tiles_r, int tiles_c) {
    // One array per stage and operand: distinct LDS objects let the compiler see that the
    // direct-to-LDS loads of one stage do not alias the fragment reads of the other, so it does
    // not make the reads wait for the loads in flight.
    __shared__ __attribute__((aligned(1024))) uint8_t ldsA0[kSlabBytes];
    __shared__ __attribute__((aligned(1024))) uint8_t ldsB0[kSlabBytes];
    __shared__ __attribute__((aligned(1024))) uint8_t ldsA1[kSlabBytes];
    __shared__ __attribute__((aligned(1024))) uint8_t ldsB1[kSlabBytes];
    __shared__ unsigned s_amax[kGemmThreads / kWave];
    int tr, tc;
    if (!tile_of_block(blockIdx.x, tiles_r, tiles_c, tr, tc)) return;   // uniform over the workgroup

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int wr = wave >> 1, wc = wave & 1;

    // ---- global -> LDS: one instruction moves 8 rows x 128 B; wave w moves rows [64w, 64w+64) of A and B
    const __amdgpu_buffer_rsrc_t rsA = make_rsrc(A + (size_t)tr * BM * T, (unsigned)((size_t)BM * T));
    const __amdgpu_buffer_rsrc_t rsB = make_rsrc(B + (size_t)tc * BN * T, (unsigned)((size_t)BN * T));
    const int ld_row = lane >> 3;                                   // row inside the group of 8
    const int ld_voff = ld_row * T + (((lane & 7) ^ ld_row) << 4);
    const int ld_soff = wave * 64 * T;
    auto issue_loads = [&](uint8_t* slabA, uint8_t* slabB, int k0) {
        uint8_t* sa = slabA + wave * 64 * BK;
        uint8_t* sb = slabB + wave * 64 * BK;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, (lds_void*)(sa + j * 8 * BK), 16, ld_voff, ld_soff + k0 + j * 8 * T, 0, 0);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB, (lds_void*)(sb + j * 8 * BK), 16, ld_voff, ld_soff + k0 + j * 8 * T, 0, 0);
        }
    };

    // ---- LDS -> registers: lane reads 32 contiguous bytes (two swizzled 16-byte chunks) of its row
    const int fr_row = lane & 31;
    const int fr_half = lane >> 5;                                  // which 32 bytes of the 64-byte K half
    const int swz = fr_row & 7;                                     // (row & 7) for every row this lane reads
    // byte offsets inside a slab for K-half 0 and 1, first and second chunk
    const int offA = (wr * 128 + fr_row) * BK, offB = (wc * 128 + fr_row) * BK;
    const int ch00 = ((fr_half * 2) ^ swz) << 4, ch01 = ((fr_half * 2 + 1) ^ swz) << 4;
    const int ch10 = ((4 + fr_half * 2) ^ swz) << 4, ch11 = ((4 + fr_half * 2 + 1) ^ swz) << 4;
    auto read_frags = [&](const uint8_t* slab, int off, int ks, v8i (&f)[4]) {
        const int c0 = ks ? ch10 : ch00, c1 = ks ? ch11 : ch01;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint8_t* p = slab + off + i * 32 * BK;
            v4i lo = *reinterpret_cast<const v4i*>(p + c0);
            v4i hi = *reinterpret_cast<const v4i*>(p + c1);
            f[i] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
    };

    v16f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    v8i a0[4], b0[4], a1[4], b1[4];        // fragment sets of the two 64-byte halves of a K step
    const int nk = T / BK;

    // One K step on the stage (curA, curB) while the other stage (nxtA, nxtB) is being filled:
    //   first half : read the second-half fragments            | 16 MFMAs on the first-half fragments
    //   barrier    : the next slab has landed, everybody is done reading the current one
    //   second half: start loading slab kt+2 into the current stage, read the first-half
    //                fragments of slab kt+1                     | 16 MFMAs on the second-half fragments
    // Loads that would start beyond the last slab are pointed outside the buffer range instead:
    // the hardware then fetches nothing, and the stage they would fill is never read.
    constexpr int kOutOfRange = 0x7FFFFF00;
    auto k_step = [&](uint8_t* curA, uint8_t* curB, uint8_t* nxtA, uint8_t* nxtB, int kt) {
        read_frags(curA, offA, 1, a1);
        read_frags(curB, offB, 1, b1);
        mma_4x4<FA, FB>(acc, a0, b0);
        // fragment reads ride along with the first 8 MFMAs, so that they have landed by the 16th
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(kSchedMfma, 1, 0);
            __builtin_amdgcn_sched_group_barrier(kSchedDsRead, 2, 0);
        }
        __builtin_amdgcn_sched_group_barrier(kSchedMfma, 8, 0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        issue_loads(curA, curB, kt + 2 < nk ? (kt + 2) * BK : kOutOfRange);
        read_frags(nxtA, offA, 0, a0);          // past the last slab this reads stale bytes that are never used
        read_frags(nxtB, offB, 0, b0);
        mma_4x4<FA, FB>(acc, a1, b1);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(kSchedMfma, 1, 1);
            __builtin_amdgcn_sched_group_barrier(kSchedDsRead, 2, 1);
            __builtin_amdgcn_sched_group_barrier(kSchedVmemRead, 1, 1);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(kSchedMfma, 1, 1);
            __builtin_amdgcn_sched_group_barrier(kSchedVmemRead, 1, 1);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    issue_loads(ldsA0, ldsB0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    issue_loads(ldsA1, ldsB1, nk > 1 ? BK : kOutOfRange);
    read_frags(ldsA0, offA, 0, a0);
    read_frags(ldsB0, offB, 0, b0);
    int kt = 0;
    for (; kt + 1 < nk; kt += 2) {
        k_step(ldsA0, ldsB0, ldsA1, ldsB1, kt);
        k_step(ldsA1, ldsB1, ldsA0, ldsB0, kt + 1);
    }
    if (kt < nk) k_step(ldsA0, ldsB0, ldsA1, ldsB1, kt);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // nothing may still be landing in LDS when the wave ends

    // ---- epilogue: lane holds, per block, 4 groups of 4 consecutive columns of row (lane % 32)
    const float inv_a = 1.0f / *d_sA, inv_b = 1.0f / *d_sB;
    unsigned mag = 0;
    const int row_base = tr * BM + wr * 128 + fr_row;
    const int col_base = tc * BN + wc * 128 + fr_half * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint16_t* crow = C + (size_t)(row_base + i * 32) * Cn + col_base;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint16_t* dst = crow + j * 32 + g * 8;
                v4f y;
#pragma unroll
                for (int e = 0; e < 4; ++e) y[e] = acc[i][j][4 * g + e] * inv_a * inv_b;
                if (accumulate) {
                    v2u old = *reinterpret_cast<const v2u*>(dst);
                    y[0] += __uint_as_float(old[0] << 16);
                    y[1] += __uint_as_float(old[0] & 0xFFFF0000u);
                    y[2] += __uint_as_float(old[1] << 16);
                    y[3] += __uint_as_float(old[1] & 0xFFFF0000u);
                }
                bf16x4 o = __builtin_convertvector(y, bf16x4);
                mag = bf16_mag_max4(mag, o);
                *reinterpret_cast<bf16x4*>(dst) = o;
            }
        }
    }
    if (amax_bits) {
        mag = wave_max_u32(mag);
        if (lane == 0) s_amax[wave] = mag;
        __syncthreads();
        if (threadIdx.x == 0) {
#pragma unroll
            for (int w = 1; w < kGemmThreads / kWave; ++w) mag = mag > s_amax[w] ? mag : s_amax[w];
            atomicMax(amax_bits, amax_bits_from_bf16_mag(mag));
        }
    }
}

// ---- generic kernel: one wavefront per 16x16 outputs, v_mfma_f32_16x16x128_f8f6f4, guarded loads
template <int FA, int FB>
__global__ __launch_bounds__(256) void gemm_tn_generic_kernel(
    const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, uint16_t* __restrict__ C,
    int64_t R, int64_t Cn, int64_t T, const float* __restrict__ d_sA, const float* __restrict__ d_sB,
    int accumulate, unsigned* __restrict__ amax_bits) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t r0 = ((int64_t)blockIdx.y * 2 + (wave >> 1)) * 16;
    const int64_t c0 = ((int64_t)blockIdx.x * 2 + (wave & 1)) * 16;
    const int64_t ar = r0 + (lane & 15), bc = c0 + (lane & 15);
    const bool a_ok = ar < R, b_ok = bc < Cn;
    const bool vec_ok = (T % 16) == 0;
    auto load32 = [&](const uint8_t* base, bool ok, int64_t row, int64_t k) -> v8i {
        v8i v = {0, 0, 0, 0, 0, 0, 0, 0};
        if (!ok || k >= T) return v;
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
        v8i a = load32(A, a_ok, ar, k);
        v8i b = load32(B, b_ok, bc, k);
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

__global__ void gemm_amax_reset_kernel(unsigned* amax_bits) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *amax_bits = 0u;
}

template <int FA, int FB>
static void launch_one(const uint8_t* A, const uint8_t* B, int64_t R, int64_t C, int64_t T,
                       const float* sA, const float* sB, void* c, int accumulate, unsigned* amax,
                       hipStream_t stream) {
    const bool tuned = R % BM == 0 && C % BN == 0 && T % BK == 0 &&
                       (size_t)BM * T < (1ull << 31) && R * T < (1ll << 40) && C * T < (1ll << 40);
    if (tuned) {
        const int tiles_r = (int)(R / BM), tiles_c = (int)(C / BN);
        const int nt = tiles_r * tiles_c;
        const int grid = ((nt + kXcds - 1) / kXcds) * kXcds;
        hipLaunchKernelGGL((gemm_tn_256_kernel<FA, FB>), dim3(grid), dim3(kGemmThreads), 0, stream,
                           A, B, reinterpret_cast<uint16_t*>(c), (int)C, (int)T, sA, sB,
                           accumulate, amax, tiles_r, tiles_c);
    } else {
        dim3 grid((unsigned)((C + 31) / 32), (unsigned)((R + 31) / 32));
        hipLaunchKernelGGL((gemm_tn_generic_kernel<FA, FB>), grid, dim3(256), 0, stream,
                           A, B, reinterpret_cast<uint16_t*>(c), R, C, T, sA, sB, accumulate, amax);
    }
}

int launch_gemm_tn(const uint8_t* A, int fmtA, const uint8_t* B, int fmtB, int64_t R, int64_t C,
                   int64_t T, const float* d_scaleA, const float* d_scaleB, void* c_bf16,
                   int accumulate, float* d_amax_c, hipStream_t stream, int num_cus) {
    (void)num_cus;
    unsigned* amax = reinterpret_cast<unsigned*>(d_amax_c);
    if (amax) hipLaunchKernelGGL(gemm_amax_reset_kernel, dim3(1), dim3(64), 0, stream, amax);
    if (fmtA == 0 && fmtB == 0) launch_one<0, 0>(A, B, R, C, T, d_scaleA, d_scaleB, c_bf16, accumulate, amax, stream);
    else if (fmtA == 1 && fmtB == 0) launch_one<1, 0>(A, B, R, C, T, d_scaleA, d_scaleB, c_bf16, accumulate, amax, stream);
    else if (fmtA == 0 && fmtB == 1) launch_one<0, 1>(A, B, R, C, T, d_scaleA, d_scaleB, c_bf16, accumulate, amax, stream);
    else launch_one<1, 1>(A, B, R, C, T, d_scaleA, d_scaleB, c_bf16, accumulate, amax, stream);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace llmq
