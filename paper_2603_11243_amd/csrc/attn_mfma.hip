// Causal self-attention over ragged (varlen) utterances, head_dim 128, grouped KV heads, 16-bit MFMA (IEEE half
// or bfloat16 operands: template parameter BF).
// This is the mechanism that lets Eq. 5 be evaluated for all draft tokens in one forward (Sec. 2.2):
// position p only attends to positions <= p of its own utterance.
//
// A workgroup owns 64 query positions of one (utterance, KV head): 2 x RATIO wavefronts, one per
// (query head of the group, 32-row block), so that a K/V block is staged once for every query head
// that shares it.  Keys/values are visited in blocks of 64 with an online softmax.
//   S^T[key, q]  = K . Q^T      (A operand: K rows from LDS, B operand: Q rows held in registers)
//   O^T[dim, q] += V^T . P^T    (A operand: V^T rows from LDS, B operand: P^T)
// Working with the transposed products keeps a query position in one lane column (lane%32) for
// both MFMAs, so the softmax statistics are per-lane scalars and the fp32 accumulator registers of
// S^T turn into the B operand of the second MFMA after an f16 pack, without any data exchange.
// The k-slot order of that operand is the accumulator's row order, so V^T is written to LDS with
// the keys of every group of 16 permuted the same way (bits 2 and 3 of the key index swapped).
#include "gemm_core.h"
#include "ssd_internal.h"

namespace ssd {

constexpr int ATT_HD = 128;
constexpr int ATT_KB = 64;                    // keys per block
constexpr int ATT_K_STRIDE = ATT_HD + 8;      // Ks[key][dim], elements
constexpr int ATT_V_STRIDE = ATT_KB + 8;      // Vt[dim][slot], elements
// register-resident staging values: a native vector type (struct-typed arrays that are filled under a
// condition end up in scratch memory)
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

template <int RATIO, bool BF>      // query heads per KV head; operand type (IEEE half / bfloat16)
__global__ void __launch_bounds__(128 * RATIO, 2) attn_mfma_kernel(const f16_t* __restrict__ qkv, f16_t* __restrict__ out,
                                                                const AttnTile* __restrict__ tiles, int n_q_heads,
                                                                int n_kv_heads) {
    constexpr int NT = 128 * RATIO;
    constexpr int STAGE_ITERS = (ATT_KB * 16 + NT - 1) / NT;      // 16-byte chunks of a 64 x 128 block per thread
    // LDS: the K / V^T block, and (before the first and after the last block) one 32-row staging tile per
    // wavefront through which Q comes in and O goes out, so that global memory sees whole 256-byte rows
    constexpr int KV_BYTES = (ATT_KB * ATT_K_STRIDE + ATT_HD * ATT_V_STRIDE) * 2;
    constexpr int WAVE_BYTES = 32 * ATT_K_STRIDE * 2;
    constexpr int SMEM_BYTES = KV_BYTES > 2 * RATIO * WAVE_BYTES ? KV_BYTES : 2 * RATIO * WAVE_BYTES;
    __shared__ __align__(16) unsigned char smem[SMEM_BYTES];
    f16_t* Ks = reinterpret_cast<f16_t*>(smem);
    f16_t* Vt = Ks + ATT_KB * ATT_K_STRIDE;
    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
    const int hgrp = lane / 32, lcol = lane % 32;
    // work index = tile * n_kv_heads + kv head, dealt so that one XCD walks a contiguous run: the tiles of
    // an utterance (which re-read its keys and values) then share an L2
    const int work = xcd_contiguous_index(blockIdx.x, gridDim.x);
    const AttnTile t = tiles[work / n_kv_heads];
    const int kvh = work % n_kv_heads;
    const int head = kvh * RATIO + wave / 2;
    const int d_q = n_q_heads * ATT_HD, d_kv = n_kv_heads * ATT_HD;
    const int ldq = d_q + 2 * d_kv;
    const f16_t* seq = qkv + (int64_t)t.seq_start * ldq;
    const f16_t* kbase = seq + d_q + kvh * ATT_HD;
    const f16_t* vbase = kbase + d_kv;

    const int q_first = t.q_start + (wave % 2) * 32;    // first query position of this wavefront
    const int qpos = q_first + lcol;
    const bool wave_live = q_first < t.seq_len;

    // Q^T fragments: lane supplies query row qpos, dims 16*kk + 8*hgrp .. +8.  The 32 x 128 tile is read
    // from global memory row by row (16 lanes per 256-byte row) and redistributed through LDS; the loads
    // are issued here, the redistribution follows once the first K/V loads are in flight too.
    f16_t* wtile = reinterpret_cast<f16_t*>(smem + wave * WAVE_BYTES);
    u32x4_t qrow[8] = {};
    if (wave_live) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = min(q_first + i * 4 + lane / 16, t.seq_len - 1);
            qrow[i] = *reinterpret_cast<const u32x4_t*>(seq + (int64_t)row * ldq + head * ATT_HD + (lane % 16) * 8);
        }
    }
    f32x16_t o_acc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float sc = 0.08838834764831845f * 1.4426950408889634f;   // log2(e) / sqrt(128)

    const int kv_end = min(t.seq_len, t.q_start + 64);              // keys needed by this tile
    // K/V blocks go global -> registers -> LDS; the registers of block kb+1 are loaded while block kb
    // is being multiplied.  K: thread owns (key = c/16, 8 dims) -> coalesced rows.  V: thread owns a pair
    // of neighbouring keys and 8 dims, so that it writes whole dwords of V^T (two keys of one dim).
    constexpr int PAIR_ITERS = (ATT_KB / 2 * 16 + NT - 1) / NT;
    u32x4_t k_reg[STAGE_ITERS] = {}, v_reg[PAIR_ITERS][2] = {};
    auto load_kv = [&](int kb) {
#pragma unroll
        for (int it = 0; it < STAGE_ITERS; ++it) {
            const int c = tid + it * NT;
            if (c < ATT_KB * 16) {
                const int krow = min(kb + c / 16, t.seq_len - 1);
                k_reg[it] = *reinterpret_cast<const u32x4_t*>(kbase + (int64_t)krow * ldq + (c % 16) * 8);
            }
        }
#pragma unroll
        for (int it = 0; it < PAIR_ITERS; ++it) {
            const int q = tid + it * NT;
            if (q < ATT_KB / 2 * 16) {
                const int key = kb + 2 * (q % 32), dc = q / 32;
                v_reg[it][0] = *reinterpret_cast<const u32x4_t*>(vbase + (int64_t)min(key, t.seq_len - 1) * ldq + dc * 8);
                v_reg[it][1] = *reinterpret_cast<const u32x4_t*>(vbase + (int64_t)min(key + 1, t.seq_len - 1) * ldq + dc * 8);
            }
        }
    };
    load_kv(0);
    f16x8_t qf[8];
    if (wave_live) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            *reinterpret_cast<u32x4_t*>(wtile + (i * 4 + lane / 16) * ATT_K_STRIDE + (lane % 16) * 8) = qrow[i];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
            qf[kk] = as_f16x8(*reinterpret_cast<const uint4*>(wtile + lcol * ATT_K_STRIDE + kk * 16 + hgrp * 8));
    }
    __syncthreads();                 // every wavefront has its Q fragments: the staging tiles may be overwritten
    for (int kb = 0; kb < kv_end; kb += ATT_KB) {
        // ---- stage K (row-major) and V (transposed, permuted) blocks
#pragma unroll
        for (int it = 0; it < STAGE_ITERS; ++it) {
            const int c = tid + it * NT;
            if (c < ATT_KB * 16)
                *reinterpret_cast<u32x4_t*>(Ks + (c / 16) * ATT_K_STRIDE + (c % 16) * 8) = k_reg[it];
        }
#pragma unroll
        for (int it = 0; it < PAIR_ITERS; ++it) {
            const int q = tid + it * NT;
            if (q < ATT_KB / 2 * 16) {
                const int key = 2 * (q % 32), dc = q / 32;
                const int slot = (key & ~12) | ((key & 4) << 1) | ((key & 8) >> 1);      // even; key+1 -> slot+1
                uint32_t* vd = reinterpret_cast<uint32_t*>(Vt + (dc * 8) * ATT_V_STRIDE + slot);
                const u32x4_t a = v_reg[it][0], b = v_reg[it][1];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    vd[(2 * e) * (ATT_V_STRIDE / 2)] = (a[e] & 0xffffu) | (b[e] << 16);
                    vd[(2 * e + 1) * (ATT_V_STRIDE / 2)] = (a[e] >> 16) | (b[e] & 0xffff0000u);
                }
            }
        }
        if (kb + ATT_KB < kv_end) load_kv(kb + ATT_KB);
        __syncthreads();
        if (wave_live && kb <= q_first + 31) {
            // ---- S^T for the two 32-key halves of the block.  The K fragments are read four MFMAs ahead (a read
            // issued right before its MFMA leaves the LDS latency exposed 32 times per block).
            f32x16_t s_acc[2];
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) s_acc[c][r] = 0.f;
            const f16_t* kf0 = Ks + lcol * ATT_K_STRIDE + hgrp * 8;
            auto k_frag = [&](int idx) {      // idx = 8 * half + kk
                return as_f16x8(*reinterpret_cast<const uint4*>(kf0 + (idx / 8) * 32 * ATT_K_STRIDE + (idx % 8) * 16));
            };
            f16x8_t kq[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) kq[p] = k_frag(p);
#pragma unroll
            for (int idx = 0; idx < 16; ++idx) {
                s_acc[idx / 8] = mfma_32x32x16<BF>(kq[idx % 4], qf[idx % 8], s_acc[idx / 8]);
                if (idx + 4 < 16) kq[idx % 4] = k_frag(idx + 4);
            }
            // pin the order (the scheduler would sink every read to just before its MFMA)
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
            for (int idx = 0; idx < 16; ++idx) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (idx + 4 < 16) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            // first V^T fragments: their latency hides behind the softmax arithmetic
            const f16_t* vf0 = Vt + lcol * ATT_V_STRIDE + hgrp * 8;
            auto v_frag = [&](int idx) {      // idx = 4 * db + ks
                return as_f16x8(*reinterpret_cast<const uint4*>(vf0 + (idx / 4) * 32 * ATT_V_STRIDE + (idx % 4) * 16));
            };
            f16x8_t vq[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) vq[p] = v_frag(p);
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
            // ---- causal mask (only blocks that reach past the first query of the wavefront)
            if (kb + ATT_KB - 1 > q_first) {
#pragma unroll
                for (int c = 0; c < 2; ++c)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int kpos = kb + c * 32 + 8 * (r / 4) + 4 * hgrp + (r % 4);
                        if (kpos > qpos) s_acc[c][r] = -INFINITY;
                    }
            }
            // ---- online softmax; lanes l and l^32 share a query position
            float bm = -INFINITY;
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) bm = fmaxf(bm, s_acc[c][r]);
            bm = fmaxf(bm, __shfl_xor(bm, 32));
            const float m_new = fmaxf(m_run, bm);
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * sc);
            const float ms = m_new * sc;
            float rs = 0.f;
            f16x8_t pf[4];
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    uint32_t w[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float p0 = __builtin_amdgcn_exp2f(fmaf(s_acc[c][8 * s + 2 * e], sc, -ms));
                        const float p1 = __builtin_amdgcn_exp2f(fmaf(s_acc[c][8 * s + 2 * e + 1], sc, -ms));
                        rs += p0 + p1;
                        w[e] = op_pack2<BF>(p0, p1);
                    }
                    pf[c * 2 + s] = as_f16x8(make_uint4(w[0], w[1], w[2], w[3]));
                }
            rs += __shfl_xor(rs, 32);
            l_run = l_run * alpha + rs;
            m_run = m_new;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[db][r] *= alpha;
            // ---- O^T += V^T . P^T
#pragma unroll
            for (int idx = 0; idx < 16; ++idx) {
                o_acc[idx / 4] = mfma_32x32x16<BF>(vq[idx % 4], pf[idx % 4], o_acc[idx / 4]);
                if (idx + 4 < 16) vq[idx % 4] = v_frag(idx + 4);
            }
#pragma unroll
            for (int idx = 0; idx < 16; ++idx) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (idx + 4 < 16) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        }
        __syncthreads();
    }
    // the loop ended with a barrier: K / V^T are dead, the staging tiles are free again
    if (wave_live) {
        const float inv = 1.0f / l_run;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int dim = db * 32 + 8 * g + 4 * hgrp;
                uint2 w;
                w.x = op_pack2<BF>(o_acc[db][4 * g] * inv, o_acc[db][4 * g + 1] * inv);
                w.y = op_pack2<BF>(o_acc[db][4 * g + 2] * inv, o_acc[db][4 * g + 3] * inv);
                *reinterpret_cast<uint2*>(wtile + lcol * ATT_K_STRIDE + dim) = w;
            }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = q_first + i * 4 + lane / 16;
            const uint4 w = *reinterpret_cast<const uint4*>(wtile + (i * 4 + lane / 16) * ATT_K_STRIDE + (lane % 16) * 8);
            if (row < t.seq_len)
                *reinterpret_cast<uint4*>(out + (int64_t)(t.seq_start + row) * d_q + head * ATT_HD + (lane % 16) * 8) = w;
        }
    }
}

template <bool BF>
static void attn_impl(const uint16_t* qkv, uint16_t* out, const AttnTile* tiles, int n_tiles, int n_q_heads, int n_kv_heads,
                      hipStream_t st) {
    const int ratio = n_q_heads / n_kv_heads;
    const dim3 grid(n_tiles * n_kv_heads);
    if (ratio == 1) hipLaunchKernelGGL((attn_mfma_kernel<1, BF>), grid, dim3(128), 0, st, qkv, out, tiles, n_q_heads, n_kv_heads);
    else if (ratio == 2) hipLaunchKernelGGL((attn_mfma_kernel<2, BF>), grid, dim3(256), 0, st, qkv, out, tiles, n_q_heads, n_kv_heads);
    else if (ratio == 3) hipLaunchKernelGGL((attn_mfma_kernel<3, BF>), grid, dim3(384), 0, st, qkv, out, tiles, n_q_heads, n_kv_heads);
    else hipLaunchKernelGGL((attn_mfma_kernel<4, BF>), grid, dim3(512), 0, st, qkv, out, tiles, n_q_heads, n_kv_heads);
}
void launch_attn_mfma(const uint16_t* qkv, uint16_t* out, const AttnTile* tiles, int n_tiles, int n_q_heads,
                      int n_kv_heads, bool bf16_ops, hipStream_t st) {
    if (n_tiles <= 0) return;
    if (bf16_ops) attn_impl<true>(qkv, out, tiles, n_tiles, n_q_heads, n_kv_heads, st);
    else attn_impl<false>(qkv, out, tiles, n_tiles, n_q_heads, n_kv_heads, st);
}

}  // namespace ssd
