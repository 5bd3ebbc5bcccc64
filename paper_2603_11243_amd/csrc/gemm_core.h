// 16-bit MFMA GEMM main loop for gfx950:  acc[M,N] = A[M,K] * W[N,K]^T, fp32 accumulation.
// Operands are IEEE half (f16): same matrix-core rate as bf16 on this chip, 3 more mantissa bits
// for the activations; weights stored as bf16 are converted exactly (power-of-two scale) once.
//
// Both operands are K-contiguous, which is exactly the operand layout of
// v_mfma_f32_32x32x16_f16: a lane supplies 8 consecutive k of one row (A) or one column (W row).
// Lane l of a wavefront holds, for a 32x32 accumulator block, column l%32 and rows
// 8*(r/4) + 4*(l/32) + r%4 for register r = 0..15.
//
// A workgroup of WAVES_M x WAVES_N wavefronts computes a BM x BN tile.  K is consumed in slices of
// BK = 64 (128 bytes per row) that go from global memory straight into LDS with
// buffer_load_dwordx4 ... lds (no register staging) through a ring of NSTAGE LDS stages: the loads
// of the next NSTAGE-1 slices are in flight while the MFMAs of the current slice run, one barrier
// per slice.  Big tiles use two stages (compute bound); the skinny tile for a handful of rows uses
// more, because there the job is to keep enough weight bytes in flight.
// LDS layout of a slice: row-major, 128 bytes per row, the eight 16-byte chunks of row r stored at
// chunk position c ^ ((r >> 1) & 7).  A load instruction fills 1 KB of LDS with lane i's 16 bytes at
// byte 16*i, so lane i fetches the global chunk that belongs at that position.  A fragment read
// (consecutive rows, same logical chunk) then spreads every 16 lanes over all sixteen 16-byte
// columns of the 256-byte LDS data path (measured: SQ_LDS_BANK_CONFLICT drops to zero; with
// c ^ (r & 7) half of the LDS cycles were conflict cycles).
// Rows >= M (and columns >= n_rows_w, if given) are clamped on load and must be skipped by the epilogue.
// Requirements: N % BN == 0, K % 64 == 0, A and W 16-byte aligned and smaller than 4 GiB.
#pragma once
#include <type_traits>
#include "device_utils.h"

namespace ssd {

typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void lds_void_t;

constexpr int GEMM_BK = 64;
constexpr int GEMM_ROW_BYTES = GEMM_BK * 2;

// Hardware deals consecutive workgroup ids round-robin to the 8 XCDs, each with its own L2.  This maps
// a workgroup id to a work index such that every XCD walks one contiguous run of indices, so that
// neighbouring indices (which share operand panels) meet in the same L2.
__device__ __forceinline__ int xcd_contiguous_index(int pid, int total) {
    constexpr int XCDS = 8;
    const int per = total / XCDS, rem = total % XCDS;
    const int xcd = pid % XCDS, idx = pid / XCDS;
    return (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx;
}

template <int BM, int BN, int NSTAGE = 2>
constexpr size_t gemm_lds_bytes() { return (size_t)NSTAGE * (BM + BN) * GEMM_ROW_BYTES; }

__device__ __forceinline__ f16x8_t as_f16x8(const uint4& v) { return __builtin_bit_cast(f16x8_t, v); }

// The two matrix instructions of the 16-bit path for either operand type (f16x8_t is the 16-byte container of
// eight operand bit patterns in both cases); same shapes, same rate.
typedef float f32x4_t __attribute__((ext_vector_type(4)));
template <bool BF>
__device__ __forceinline__ f32x16_t mfma_32x32x16(const f16x8_t& a, const f16x8_t& b, const f32x16_t& c) {
    if constexpr (BF) return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}
template <bool BF>
__device__ __forceinline__ f32x4_t mfma_16x16x32(const f16x8_t& a, const f16x8_t& b, const f32x4_t& c) {
    if constexpr (BF) return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// Row / column of accumulator register r of block (i, j) for this lane, relative to the wave tile.
__device__ __forceinline__ int acc_row(int i, int r, int lane) { return i * 32 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4); }
__device__ __forceinline__ int acc_col(int j, int lane) { return j * 32 + (lane % 32); }

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p) {
    // raw buffer, no bounds (offsets are clamped by the caller), data format 32 bit
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, 0xffffffff, 0x00020000);
}

// BF16 = true: the operands are bfloat16 bit patterns and the bf16 MFMA is used (same shapes and rate).
template <int BM, int BN, int WAVES_M, int WAVES_N, int NSTAGE = 2, bool BF16 = false>
struct GemmTile {
    static constexpr int WAVES = WAVES_M * WAVES_N;
    static constexpr int NT = 64 * WAVES;
    static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    static constexpr int TM = WTM / 32, TN = WTN / 32;
    static constexpr int A_LOADS = BM / (8 * WAVES);     // 1 KB (8 rows) per wavefront load instruction
    static constexpr int B_LOADS = BN / (8 * WAVES);
    static constexpr int A_BYTES = BM * GEMM_ROW_BYTES, B_BYTES = BN * GEMM_ROW_BYTES;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static_assert(BM % (8 * WAVES) == 0 && BN % (8 * WAVES) == 0, "tile/thread mismatch");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of 32x32");

    // acc is accumulated onto (zero it for a plain product).  Rows of W at and beyond n_rows_w are
    // clamped on load like the rows of A beyond M (for callers whose ragged dimension is N).  smem: gemm_lds_bytes<BM,BN,NSTAGE>() bytes, 16-byte
    // aligned.  Slices kt0 <= kt < kt1 of K are accumulated (K itself is the row stride of A and W).
    static __device__ __forceinline__ void run(const f16_t* __restrict__ A, const f16_t* __restrict__ W, int M, int K,
                                               int m0, int n0, int kt0, int kt1, unsigned char* smem,
                                               f32x16_t (&acc)[TM][TN], int n_rows_w = 0x7fffffff, int lda = 0, int ldw = 0) {
        if (lda == 0) lda = K;                               // row strides in elements (default: dense rows)
        if (ldw == 0) ldw = K;
        // Wavefronts beyond WAVES form further groups of WAVES that run the same tile on their own smem and K range
        // (in-workgroup K split: the caller adds the groups' accumulators); every group must run the same number
        // of slices, since the barriers below are workgroup barriers.
        const int tid = threadIdx.x, lane = tid % 64;
        const int wave = __builtin_amdgcn_readfirstlane((tid / 64) % WAVES);
        const int wm = wave / WAVES_N, wn = wave % WAVES_N;
        const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(A), w_rsrc = make_rsrc(W);

        // ---- global -> LDS: byte offsets of this lane's chunk for every load instruction
        // instruction i of this wavefront fills rows (i*WAVES + wave)*8 .. +7 of the slice
        const int lrow = lane / 8, lslot = lane % 8;            // position inside the 1 KB block
        unsigned a_off[A_LOADS], b_off[B_LOADS];
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) {
            const int r = (i * WAVES + wave) * 8 + lrow;
            const int grow = min(m0 + r, M - 1);
            a_off[i] = (unsigned)grow * (unsigned)lda * 2u + (unsigned)((lslot ^ ((r >> 1) & 7)) * 16);
        }
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i) {
            const int r = (i * WAVES + wave) * 8 + lrow;
            b_off[i] = (unsigned)min(n0 + r, n_rows_w - 1) * (unsigned)ldw * 2u + (unsigned)((lslot ^ ((r >> 1) & 7)) * 16);
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

        // ---- LDS -> fragments: row = lane%32 (+32 per block), logical chunk = 2*kk + lane/32
        int a_rd[GEMM_BK / 16], b_rd[GEMM_BK / 16];
#pragma unroll
        for (int kk = 0; kk < GEMM_BK / 16; ++kk) {
            const int slot = (2 * kk + lane / 32) ^ ((lane >> 1) & 7);
            a_rd[kk] = (wm * WTM + lane % 32) * GEMM_ROW_BYTES + slot * 16;
            b_rd[kk] = A_BYTES + (wn * WTN + lane % 32) * GEMM_ROW_BYTES + slot * 16;
        }

        auto read_frags = [&](int stage, int kk, f16x8_t (&a)[TM], f16x8_t (&b)[TN]) {
            const unsigned char* sbase = smem + stage * STAGE_BYTES;
#pragma unroll
            for (int i = 0; i < TM; ++i)
                a[i] = as_f16x8(*reinterpret_cast<const uint4*>(sbase + a_rd[kk] + i * 32 * GEMM_ROW_BYTES));
#pragma unroll
            for (int j = 0; j < TN; ++j)
                b[j] = as_f16x8(*reinterpret_cast<const uint4*>(sbase + b_rd[kk] + j * 32 * GEMM_ROW_BYTES));
        };
        auto mfma_block = [&](const f16x8_t (&a)[TM], const f16x8_t (&b)[TN]) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = mfma_32x32x16<BF16>(a[i], b[j], acc[i][j]);
        };

        // Software pipeline over n = kt1 - kt0 slices; slice i lives in stage i % NSTAGE.
        // Invariant at the top of iteration i: slice i has landed, its kk=0 fragments are in (a0, b0),
        // slices i+1 .. i+NSTAGE-1 are in flight.  The fragments of step kk+1 are read while the
        // MFMAs of step kk run; the barrier that ends a slice sits between the last fragment read
        // and the last MFMA block, so the first fragment read of the next slice and the global
        // loads that refill the freed stage are issued before that MFMA block and overlap with it.
        constexpr int KK = GEMM_BK / 16;
        constexpr int HALF = TM * TN / 2;
        constexpr int LOADS_PER_MFMA = (A_LOADS + B_LOADS + HALF - 1) / HALF;
        constexpr int READS_PER_MFMA = (TM + TN + HALF - 1) / HALF;
        static_assert(KK == 4, "pipeline below is written for four k-steps per slice");
        static_assert(NSTAGE >= 2 && (NSTAGE - 2) * (A_LOADS + B_LOADS) <= 63, "vmcnt range");
        // s_waitcnt immediates: lgkmcnt(0) with vmcnt(V): V low 4 bits in [3:0], high 2 bits in [15:14]
        constexpr int V_KEEP = (NSTAGE - 2) * (A_LOADS + B_LOADS);     // loads of the younger slices may stay out
        constexpr int WAIT_KEEP = 0x0070 | (V_KEEP & 15) | ((V_KEEP >> 4) << 14);
        constexpr int WAIT_KEEP_NO_LGKM = WAIT_KEEP | 0x0F00;
        const int n = kt1 - kt0;
        f16x8_t a0[TM], b0[TN], a1[TM], b1[TN];
#pragma unroll
        for (int s = 0; s < NSTAGE; ++s)
            if (s < n) issue_loads(kt0 + s, s);
        if (n >= NSTAGE) __builtin_amdgcn_s_waitcnt(WAIT_KEEP_NO_LGKM); else __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        read_frags(0, 0, a0, b0);
        // The compiler's scheduler would sink every fragment read to just before its first use; the
        // pattern below pins "one MFMA, one LDS read" so that the reads of step kk+1 are spread under
        // the MFMAs of step kk.
        auto interleave = [&]() {
#pragma unroll
            for (int q = 0; q < TM * TN; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                 // one MFMA
                if (q < TM + TN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); // one DS read
            }
        };
        // One slice.  STEADY: the slice NSTAGE ahead exists, so the refill loads and the first fragment
        // read of the next slice are unconditional and sit in one basic block with the last MFMA
        // block, where the pattern spreads them: issued as one burst by every wavefront right after
        // the barrier, the loads queue up in the address path and hold back the MFMAs behind them.
        int stage = 0;
        auto slice = [&](auto steady, int i) {
            constexpr bool STEADY = decltype(steady)::value;
            __builtin_amdgcn_sched_barrier(0);
            read_frags(stage, 1, a1, b1);
            mfma_block(a0, b0);
            interleave();
            __builtin_amdgcn_sched_barrier(0);
            read_frags(stage, 2, a0, b0);
            mfma_block(a1, b1);
            interleave();
            __builtin_amdgcn_sched_barrier(0);
            read_frags(stage, 3, a1, b1);
            mfma_block(a0, b0);
            interleave();
            __builtin_amdgcn_sched_barrier(0);
            // all reads of `stage` are issued; wait for them and for slice i+1 (its loads are the oldest)
            const int next = (stage + 1 == NSTAGE) ? 0 : stage + 1;
            if constexpr (STEADY) {
                __builtin_amdgcn_s_waitcnt(WAIT_KEEP);
                __syncthreads();
                issue_loads(kt0 + i + NSTAGE, stage);
                read_frags(next, 0, a0, b0);
                mfma_block(a1, b1);
#pragma unroll
                for (int q = 0; q < TM * TN; ++q) {     // loads under the first half, fragment reads under the second
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    if (q < HALF) __builtin_amdgcn_sched_group_barrier(0x010, LOADS_PER_MFMA, 0);
                    else __builtin_amdgcn_sched_group_barrier(0x100, READS_PER_MFMA, 0);
                }
            } else {
                if (i + NSTAGE < n + 1) __builtin_amdgcn_s_waitcnt(WAIT_KEEP); else __builtin_amdgcn_s_waitcnt(0x0070);
                __syncthreads();
                if (i + 1 < n) read_frags(next, 0, a0, b0);
                mfma_block(a1, b1);
            }
            stage = next;
        };
        int i = 0;
        for (; i + NSTAGE < n; ++i) slice(std::true_type(), i);
        for (; i < n; ++i) slice(std::false_type(), i);
    }
};

}  // namespace ssd
