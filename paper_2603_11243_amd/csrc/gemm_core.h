// 16-bit MFMA GEMM main loop for gfx950:  acc[M,N] = A[M,K] * W[N,K]^T, fp32 accumulation.
// Operands are IEEE half (f16): same matrix-core rate as bf16 on this chip, 3 more mantissa bits
// for the activations; weights stored as bf16 are converted exactly (power-of-two scale) once.
//
// Both operands are K-contiguous, which is exactly the operand layout of
// v_mfma_f32_32x32x16_f16: a lane supplies 8 consecutive k of one row (A) or one column (W row).
// Lane l of a wavefront holds, for a 32x32 accumulator block, column l%32 and rows
// 8*(r/4) + 4*(l/32) + r%4 for register r = 0..15.
//
// A workgroup of WAVES_M x WAVES_N wavefronts computes a BM x BN tile; K is consumed in slices of
// BK = 64 staged through LDS (row stride padded to 72 elements so that the 16-byte fragment reads of
// 32 consecutive rows fall on distinct banks).  Global loads of the next slice are issued before
// the MFMAs of the current one.  Rows >= M are clamped on load and must be skipped by the epilogue.
// Requirements: N % BN == 0, K % 64 == 0, A and W 16-byte aligned.
#pragma once
#include "device_utils.h"

namespace ssd {

typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int GEMM_BK = 64;
constexpr int GEMM_LDS_STRIDE = GEMM_BK + 8;   // elements

template <int BM, int BN>
constexpr size_t gemm_lds_bytes() { return (size_t)(BM + BN) * GEMM_LDS_STRIDE * 2; }

__device__ __forceinline__ f16x8_t as_f16x8(const uint4& v) { return __builtin_bit_cast(f16x8_t, v); }

// Row / column of accumulator register r of block (i, j) for this lane, relative to the wave tile.
__device__ __forceinline__ int acc_row(int i, int r, int lane) { return i * 32 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4); }
__device__ __forceinline__ int acc_col(int j, int lane) { return j * 32 + (lane % 32); }

template <int BM, int BN, int WAVES_M, int WAVES_N>
struct GemmTile {
    static constexpr int NT = 64 * WAVES_M * WAVES_N;
    static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    static constexpr int TM = WTM / 32, TN = WTN / 32;
    static constexpr int A_CHUNKS = BM * (GEMM_BK / 8) / NT;    // 16-byte chunks per thread per slice
    static constexpr int B_CHUNKS = BN * (GEMM_BK / 8) / NT;
    static_assert(BM * (GEMM_BK / 8) % NT == 0 && BN * (GEMM_BK / 8) % NT == 0, "tile/thread mismatch");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of 32x32");

    // acc must be zero-initialised by the caller.  smem: gemm_lds_bytes<BM,BN>() bytes.
    static __device__ __forceinline__ void run(const f16_t* __restrict__ A, const f16_t* __restrict__ W, int M, int K,
                                               int m0, int n0, f16_t* smem, f32x16_t (&acc)[TM][TN]) {
        f16_t* As = smem;
        f16_t* Bs = smem + BM * GEMM_LDS_STRIDE;
        const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
        const int wm = wave / WAVES_N, wn = wave % WAVES_N;

        const uint4* a_src[A_CHUNKS];
        const uint4* b_src[B_CHUNKS];
        int a_dst[A_CHUNKS], b_dst[B_CHUNKS];
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            const int c = tid + i * NT, row = c / 8, kc = c % 8;
            const int grow = min(m0 + row, M - 1);
            a_src[i] = reinterpret_cast<const uint4*>(A + (int64_t)grow * K + kc * 8);
            a_dst[i] = row * GEMM_LDS_STRIDE + kc * 8;
        }
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) {
            const int c = tid + i * NT, row = c / 8, kc = c % 8;
            b_src[i] = reinterpret_cast<const uint4*>(W + (int64_t)(n0 + row) * K + kc * 8);
            b_dst[i] = row * GEMM_LDS_STRIDE + kc * 8;
        }
        uint4 a_reg[A_CHUNKS], b_reg[B_CHUNKS];
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) a_reg[i] = a_src[i][0];
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) b_reg[i] = b_src[i][0];

        const int a_frag = (wm * WTM + lane % 32) * GEMM_LDS_STRIDE + (lane / 32) * 8;
        const int b_frag = (wn * WTN + lane % 32) * GEMM_LDS_STRIDE + (lane / 32) * 8;
        const int KT = K / GEMM_BK;
        for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
            for (int i = 0; i < A_CHUNKS; ++i) *reinterpret_cast<uint4*>(As + a_dst[i]) = a_reg[i];
#pragma unroll
            for (int i = 0; i < B_CHUNKS; ++i) *reinterpret_cast<uint4*>(Bs + b_dst[i]) = b_reg[i];
            __syncthreads();
            if (kt + 1 < KT) {
                const int off = (kt + 1) * (GEMM_BK / 8);     // in uint4 units
#pragma unroll
                for (int i = 0; i < A_CHUNKS; ++i) a_reg[i] = a_src[i][off];
#pragma unroll
                for (int i = 0; i < B_CHUNKS; ++i) b_reg[i] = b_src[i][off];
            }
#pragma unroll
            for (int kk = 0; kk < GEMM_BK / 16; ++kk) {
                f16x8_t a[TM], b[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    a[i] = as_f16x8(*reinterpret_cast<const uint4*>(As + a_frag + i * 32 * GEMM_LDS_STRIDE + kk * 16));
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    b[j] = as_f16x8(*reinterpret_cast<const uint4*>(Bs + b_frag + j * 32 * GEMM_LDS_STRIDE + kk * 16));
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
            }
            __syncthreads();
        }
    }
};

}  // namespace ssd
