// Weight-streaming GEMM for at most 32 rows (the auto-regressive steps, the last rows of a short utterance):
//   acc[M,64] = A[M,K] * W[n0 .. n0+63, K]^T.
// With so few rows the projection is one pass over the weight matrix, and what bounds it is the number
// of weight bytes a compute unit keeps in flight and the number of cache lines a load instruction
// touches.  W is therefore read from a second copy of the weights in "stream layout": the operand
// fragments of v_mfma_f32_32x32x16_f16 stored in the order the lanes consume them, so that every load
// instruction of a wavefront is one contiguous KB and goes straight into the MFMA operand registers
// (no LDS staging, no transposition).  All loads of a wavefront's K range (up to DEPTH steps of 64) are
// issued before its first MFMA.
//
// Stream layout of W[N,K] (N % 64 == 0, K % 64 == 0), in 16-byte units of eight f16:
//   unit(T, t, j, s, h, x) = ((T * K/64 + t) * 8 + j * 4 + s) * 64 + h * 32 + x
//   holds W[64 T + 32 j + x][64 t + 32 h + 8 s .. + 7]
// (column tile T, K step t, 32-column block j, MFMA step s, lane = 32 h + x).  The MFMA wants from lane
// (x, h) eight consecutive k of column x; which eight is free as long as A and W agree, and A is read
// from LDS with the same assignment k = 64 t + 32 h + 8 s .. + 7.
//
// Work split: a workgroup owns 64 output columns and the K range of one split; its NW wavefronts take
// consecutive, equally long pieces of that range and each accumulates a full 32 x 64 partial product;
// the partial products are added through LDS in a fixed order (deterministic) by wavefront 0, which
// applies the epilogue.  A (a few KB per wavefront, L2 resident) is staged in a wavefront-private LDS
// region with the same swizzled row layout as the big GEMM (gemm_core.h), so no workgroup barrier is
// needed before the reduction.
// Requirements: (K / 64) % (splits * NW) == 0, A and W 16-byte aligned, A smaller than 4 GiB.
#pragma once
#include "gemm_core.h"

namespace ssd {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int STREAM_STEP_UNITS = 8 * 64;          // 16-byte units of one (column tile, K step) block of W

template <int NW, int DEPTH>
constexpr size_t gemm_stream_lds_bytes() {
    return (size_t)NW * (DEPTH * 4096 > 8192 ? DEPTH * 4096 : 8192);
}

template <int NW, int DEPTH, bool BF, class Epi>
__global__ void __launch_bounds__(64 * NW)
gemm_stream_kernel(const f16_t* __restrict__ A, const u32x4_t* __restrict__ Ws, int M, int N, int K, int splits, Epi epi) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    constexpr int WAVE_LDS = DEPTH * 4096 > 8192 ? DEPTH * 4096 : 8192;
    const int lane = threadIdx.x % 64;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    const int x = lane % 32, h = lane / 32;
    const int tile = blockIdx.x / splits, split = blockIdx.x % splits;
    const int KT = K / 64;
    const int steps = KT / (splits * NW);                    // K steps of this wavefront
    const int t_first = (split * NW + wave) * steps;
    unsigned char* my_lds = smem_raw + wave * WAVE_LDS;

    // A: global -> LDS, four 1 KB instructions per K step (eight rows of 128 bytes each)
    const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(A);
    const int lrow = lane / 8, lslot = lane % 8;
    unsigned a_off[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int r = q * 8 + lrow;
        a_off[q] = (unsigned)min(r, M - 1) * (unsigned)K * 2u + (unsigned)((lslot ^ ((r >> 1) & 7)) * 16);
    }
    int a_rd[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) a_rd[s] = x * GEMM_ROW_BYTES + (((4 * h + s) ^ ((x >> 1) & 7)) * 16);
    const u32x4_t* w_base = Ws + ((int64_t)tile * KT + t_first) * STREAM_STEP_UNITS + lane;

    f32x16_t acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

    for (int t0 = 0; t0 < steps; t0 += DEPTH) {
        if (t0 > 0) {                                        // fragment reads of the previous batch are done
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_void_t*)(my_lds + d * 4096 + q * 1024), 16, a_off[q],
                                                         (t_first + t0 + d) * GEMM_ROW_BYTES, 0, 0);
        // keep the issue order A, then W: the wait below counts on it
        __builtin_amdgcn_sched_barrier(0);
        u32x4_t w[DEPTH][2][4];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    w[d][j][s] = __builtin_nontemporal_load(w_base + (int64_t)(t0 + d) * STREAM_STEP_UNITS + (j * 4 + s) * 64);
        // the A loads are the oldest: wait for them only (8 DEPTH weight loads may stay in flight)
        __builtin_amdgcn_s_waitcnt(0x0F70 | ((8 * DEPTH) & 15) | (((8 * DEPTH) >> 4) << 14));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const f16x8_t a = as_f16x8(*reinterpret_cast<const uint4*>(my_lds + d * 4096 + a_rd[s]));
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[j] = mfma_32x32x16<BF>(a, __builtin_bit_cast(f16x8_t, w[d][j][s]), acc[j]);
            }
    }

    // ---- add the NW partial products in wavefront order: red[wave][j][r/4][lane] float4
    __syncthreads();                                         // every wavefront is done with its A region
    float4* red = reinterpret_cast<float4*>(smem_raw);
    if (wave != 0) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                red[(wave * 8 + j * 4 + g) * 64 + lane] = make_float4(acc[j][4 * g], acc[j][4 * g + 1], acc[j][4 * g + 2], acc[j][4 * g + 3]);
    }
    __syncthreads();
    if (wave != 0) return;
    f32x16_t out[1][2];
    out[0][0] = acc[0];
    out[0][1] = acc[1];
#pragma unroll 2
    for (int w = 1; w < NW; ++w) {                           // few at a time: the reads of one w are 32 registers
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 v = red[(w * 8 + j * 4 + g) * 64 + lane];
                out[0][j][4 * g] += v.x; out[0][j][4 * g + 1] += v.y; out[0][j][4 * g + 2] += v.z; out[0][j][4 * g + 3] += v.w;
            }
    }
    if constexpr (Epi::WANTS_SPLIT)
        epi.template operator()<1, 2>(out, 0, tile * 64, M, lane, split);
    else
        epi.template operator()<1, 2>(out, 0, tile * 64, M, lane);
}

// Row-major W[N,K] (f16) -> stream layout; one thread per 16-byte unit.
__global__ void __launch_bounds__(256) stream_layout_kernel(const u32x4_t* __restrict__ w, u32x4_t* __restrict__ out, int N, int K) {
    const int64_t n_units = (int64_t)N * K / 8;
    const int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (u >= n_units) return;
    const int KT = K / 64;
    const int xx = (int)(u % 32), hh = (int)((u / 32) % 2), ss = (int)((u / 64) % 4), jj = (int)((u / 256) % 2);
    const int64_t blk = u / STREAM_STEP_UNITS;
    const int t = (int)(blk % KT);
    const int64_t T = blk / KT;
    const int64_t row = T * 64 + jj * 32 + xx;
    out[u] = w[row * (K / 8) + 8 * t + 4 * hh + ss];
}

}  // namespace ssd
