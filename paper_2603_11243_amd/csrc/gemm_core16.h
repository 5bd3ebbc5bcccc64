// Main loop of the big-tile GEMM on v_mfma_f32_16x16x32_f16:  acc[M,N] = A[M,K] * W[N,K]^T, fp32 accumulation.
//
// Same tiling, LDS ring and global -> LDS loads as gemm_core.h (which keeps the 32x32x16 instruction for
// the skinny tiles, the LM head and the CTC output layer); only the matrix instruction and with it the
// fragment and accumulator layouts differ.  Why a second instruction shape: on this chip the big GEMMs
// run against the power limit, and the 16x16x32 shape moves half as many accumulator registers per
// flop (a 16x16 block of fp32 is read and written once per 32 k instead of a 32x32 block once per 16 k).
// A loop of nothing but independent MFMAs on random register operands sustains about 16 % more flop/s
// with it (1.79 against 1.54 PFLOP/s, two wavefronts per SIMD).
//
// Fragment layout of v_mfma_f32_16x16x32_f16: lane l supplies eight consecutive k of row (A) or
// column (W row) l % 16, namely k = 8 (l / 16) .. + 7 of the 32-wide step; of the 16x16 accumulator
// block it holds column l % 16 and rows 4 (l / 16) + r in register r = 0..3.
// A 64-wide K slice is two such steps.  A wavefront tile of WTM x WTN is (WTM/16) x (WTN/16) blocks; the
// A fragments of a step are read in two halves (upper and lower row blocks), so that the pipeline has
// four phases per slice like the 32x32x16 loop and 16 fragments live at a time:
//   phase (s, lower): MFMAs of the lower row blocks of step s   | reads: upper A fragments of step s
//   phase (s, upper): MFMAs of the upper row blocks of step s   | reads: lower A and all W fragments of step s+1
// The barrier that ends a slice sits before the last phase, which also issues the refill loads.
#pragma once
#include "gemm_core.h"

namespace ssd {


// Row / column of accumulator register r of 16x16 block (i, j) for this lane, relative to the wave tile.
struct Layout16 {
    static constexpr bool TRANSPOSED = false;
    static constexpr int BLOCK = 16, REGS = 4, PAIR = 2;     // PAIR: blocks between a column and the one 32 further
    typedef f32x4_t vec_t;
    static __device__ __forceinline__ int row(int i, int r, int lane) { return i * 16 + 4 * (lane / 16) + r; }
    static __device__ __forceinline__ int col(int j, int lane) { return j * 16 + (lane % 16); }
};
// Transposed 16x16 blocks: the MFMA is issued with the operands swapped (W fragment as the row operand), so a lane
// holds ONE row (lane % 16 of the block) and FOUR CONSECUTIVE columns 4 (lane / 16) + r.  In row-major output that
// is one 16-byte (fp32) or 8-byte (half) access per lane and block instead of four 4- or 2-byte ones: the epilogues
// issue a quarter of the memory instructions.
struct Layout16T {
    static constexpr int BLOCK = 16, REGS = 4, PAIR = 2;
    static constexpr bool TRANSPOSED = true;
    typedef f32x4_t vec_t;
    static __device__ __forceinline__ int row(int i, int lane) { return i * 16 + (lane % 16); }
    static __device__ __forceinline__ int col4(int j, int lane) { return j * 16 + 4 * (lane / 16); }    // first of four
};
struct Layout32 {
    static constexpr bool TRANSPOSED = false;
    static constexpr int BLOCK = 32, REGS = 16, PAIR = 1;
    typedef f32x16_t vec_t;
    static __device__ __forceinline__ int row(int i, int r, int lane) { return acc_row(i, r, lane); }
    static __device__ __forceinline__ int col(int j, int lane) { return acc_col(j, lane); }
};

// SWAP: issue the MFMA with the W fragment as the row operand, which transposes every accumulator block
// (Layout16T instead of Layout16); the loop, the fragments and their reads are the same.
template <int BM, int BN, int WAVES_M, int WAVES_N, bool BF16 = false, bool SWAP = false>
struct GemmTile16 {
    static constexpr int NSTAGE = 2;
    static constexpr int WAVES = WAVES_M * WAVES_N;
    static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    static constexpr int TM = WTM / 16, TN = WTN / 16;
    static constexpr int TH = TM / 2;                        // row blocks per half
    static constexpr int A_LOADS = BM / (8 * WAVES);         // 1 KB (8 rows) per wavefront load instruction
    static constexpr int B_LOADS = BN / (8 * WAVES);
    static constexpr int A_BYTES = BM * GEMM_ROW_BYTES, B_BYTES = BN * GEMM_ROW_BYTES;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static_assert(BM % (8 * WAVES) == 0 && BN % (8 * WAVES) == 0, "tile/thread mismatch");
    static_assert(WTM % 32 == 0 && WTN % 16 == 0, "wave tile: an even number of 16-row blocks, 16-column blocks");

    // acc is accumulated onto.  smem: gemm_lds_bytes<BM,BN,2>() bytes, 16-byte aligned.  K slices kt0 <= kt < kt1.
    static __device__ __forceinline__ void run(const f16_t* __restrict__ A, const f16_t* __restrict__ W, int M, int K,
                                               int m0, int n0, int kt0, int kt1, unsigned char* smem,
                                               f32x4_t (&acc)[TM][TN]) {
        const int tid = threadIdx.x, lane = tid % 64;
        const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
        const int wm = wave / WAVES_N, wn = wave % WAVES_N;
        const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(A), w_rsrc = make_rsrc(W);

        // ---- global -> LDS (identical to gemm_core.h): instruction i of this wavefront fills rows (i*WAVES + wave)*8 .. +7
        const int lrow = lane / 8, lslot = lane % 8;
        unsigned a_off[A_LOADS], b_off[B_LOADS];
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) {
            const int r = (i * WAVES + wave) * 8 + lrow;
            a_off[i] = (unsigned)min(m0 + r, M - 1) * (unsigned)K * 2u + (unsigned)((lslot ^ ((r >> 1) & 7)) * 16);
        }
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i) {
            const int r = (i * WAVES + wave) * 8 + lrow;
            b_off[i] = (unsigned)(n0 + r) * (unsigned)K * 2u + (unsigned)((lslot ^ ((r >> 1) & 7)) * 16);
        }
        auto issue_loads = [&](int kt, int stage) {
            unsigned char* sa = smem + stage * STAGE_BYTES;
            unsigned char* sb = sa + A_BYTES;
            const int koff = kt * GEMM_ROW_BYTES;
#pragma unroll
            for (int i = 0; i < A_LOADS; ++i)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_void_t*)(sa + (i * WAVES + wave) * 1024), 16, a_off[i], koff, 0, 0);
#pragma unroll
            for (int i = 0; i < B_LOADS; ++i)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(w_rsrc, (lds_void_t*)(sb + (i * WAVES + wave) * 1024), 16, b_off[i], koff, 0, 0);
        };

        // ---- LDS -> fragments: row = lane%16 (+16 per block), logical chunk = 4*s + lane/16.  Sixteen
        // consecutive rows with one logical chunk fall on sixteen different 16-byte columns (same swizzle).
        int a_rd[2], b_rd[2];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int slot = (4 * s + lane / 16) ^ (((lane % 16) >> 1) & 7);
            a_rd[s] = (wm * WTM + lane % 16) * GEMM_ROW_BYTES + slot * 16;
            b_rd[s] = A_BYTES + (wn * WTN + lane % 16) * GEMM_ROW_BYTES + slot * 16;
        }
        auto read_a = [&](int stage, int s, int half, f16x8_t (&a)[TH]) {
            const unsigned char* sbase = smem + stage * STAGE_BYTES + a_rd[s] + half * TH * 16 * GEMM_ROW_BYTES;
#pragma unroll
            for (int i = 0; i < TH; ++i) a[i] = as_f16x8(*reinterpret_cast<const uint4*>(sbase + i * 16 * GEMM_ROW_BYTES));
        };
        auto read_b = [&](int stage, int s, f16x8_t (&b)[TN]) {
            const unsigned char* sbase = smem + stage * STAGE_BYTES + b_rd[s];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = as_f16x8(*reinterpret_cast<const uint4*>(sbase + j * 16 * GEMM_ROW_BYTES));
        };
        auto mfma_half = [&](int half, const f16x8_t (&a)[TH], const f16x8_t (&b)[TN]) {
#pragma unroll
            for (int i = 0; i < TH; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[half * TH + i][j] = SWAP ? mfma_16x16x32<BF16>(b[j], a[i], acc[half * TH + i][j])
                                                 : mfma_16x16x32<BF16>(a[i], b[j], acc[half * TH + i][j]);
        };
        // scheduling patterns: one MFMA, one LDS read, for the first n_reads MFMAs of a phase
        constexpr int PH = TH * TN;                          // MFMAs per phase
        auto interleave_reads = [&](auto n_reads_c) {
            constexpr int NR = decltype(n_reads_c)::value;
#pragma unroll
            for (int q = 0; q < PH; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (q < NR) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        };
        constexpr int NL = A_LOADS + B_LOADS;
        constexpr int HALF = PH / 2;
        constexpr int LOADS_PER_MFMA = (NL + HALF - 1) / HALF;
        constexpr int READS_PER_MFMA = (TH + TN + HALF - 1) / HALF;

        const int n = kt1 - kt0;
        f16x8_t alo[TH], ahi[TH], b0[TN], b1[TN];
#pragma unroll
        for (int s = 0; s < NSTAGE; ++s)
            if (s < n) issue_loads(kt0 + s, s);
        if (n >= NSTAGE) __builtin_amdgcn_s_waitcnt(0x0F70 | (NL & 15) | ((NL >> 4) << 14)); else __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        read_a(0, 0, 0, alo);
        read_b(0, 0, b0);

        int stage = 0;
        auto slice = [&](auto steady, int i) {
            constexpr bool STEADY = decltype(steady)::value;
            __builtin_amdgcn_sched_barrier(0);
            read_a(stage, 0, 1, ahi);                        // phase (0, lower)
            mfma_half(0, alo, b0);
            interleave_reads(std::integral_constant<int, TH>());
            __builtin_amdgcn_sched_barrier(0);
            read_a(stage, 1, 0, alo);                        // phase (0, upper)
            read_b(stage, 1, b1);
            mfma_half(1, ahi, b0);
            interleave_reads(std::integral_constant<int, TH + TN>());
            __builtin_amdgcn_sched_barrier(0);
            read_a(stage, 1, 1, ahi);                        // phase (1, lower)
            mfma_half(0, alo, b1);
            interleave_reads(std::integral_constant<int, TH>());
            __builtin_amdgcn_sched_barrier(0);
            // all reads of `stage` are issued; wait for them and for slice i+1 (its loads are the oldest)
            const int next = 1 - stage;
            __builtin_amdgcn_s_waitcnt(0x0070);
            __syncthreads();
            if constexpr (STEADY) {                          // phase (1, upper) with the refill and the next slice's first reads
                issue_loads(kt0 + i + NSTAGE, stage);
                read_a(next, 0, 0, alo);
                read_b(next, 0, b0);
                mfma_half(1, ahi, b1);
#pragma unroll
                for (int q = 0; q < PH; ++q) {               // loads under the first half, fragment reads under the second
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    if (q < HALF) __builtin_amdgcn_sched_group_barrier(0x010, LOADS_PER_MFMA, 0);
                    else __builtin_amdgcn_sched_group_barrier(0x100, READS_PER_MFMA, 0);
                }
            } else {
                if (i + 1 < n) { read_a(next, 0, 0, alo); read_b(next, 0, b0); }
                mfma_half(1, ahi, b1);
            }
            stage = next;
        };
        int i = 0;
        for (; i + NSTAGE < n; ++i) slice(std::true_type(), i);
        for (; i < n; ++i) slice(std::false_type(), i);
    }
};

}  // namespace ssd
