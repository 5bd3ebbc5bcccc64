// Causal self-attention over ragged (varlen) utterances, head_dim 128, grouped KV heads, 16-bit MFMA (IEEE half
// or bfloat16 operands: template parameter BF).
// This is the mechanism that lets Eq. 5 be evaluated for all draft tokens in one forward (Sec. 2.2):
// position p only attends to positions <= p of its own utterance.
//
// A workgroup owns 64 query positions of one (utterance, query head): two wavefronts of 32 rows each.  The
// sequences of this workload are short (tens to a few hundred positions, one to a few key blocks per tile), so a
// workgroup spends most of its life waiting for its first loads and at its barriers; what counts is how many
// independent workgroups a CU holds.  Small workgroups with 32 KB of LDS and nothing staged in registers give four
// per CU; the query heads that share a KV head run next to each other on one XCD and find its keys and values in
// that XCD's L2.  Keys/values are visited in blocks of 64 with an online softmax.
//   S^T[key, q]  = K . Q^T      (A operand: K rows from LDS, B operand: Q rows held in registers)
//   O^T[dim, q] += V^T . P^T    (A operand: V^T from LDS, B operand: P^T)
// Working with the transposed products keeps a query position in one lane column (lane%32) for
// both MFMAs, so the softmax statistics are per-lane scalars and the fp32 accumulator registers of
// S^T turn into the B operand of the second MFMA after a 16-bit pack, without any data exchange.
//
// K and V blocks go global -> LDS directly (buffer_load ... lds, 1 KB = four 256-byte rows per instruction), both
// row-major with their 16-byte chunks XOR-swizzled so that every read below is free of bank conflicts:
//   K: chunk ^ (row & 15); a fragment read (ds_read_b128) touches 16 rows x one logical chunk per cycle.
//   V: chunk ^ ((row & 3) << 2); the A operand of the second MFMA needs, per lane, one dim and 8 keys, i.e. a
//      column of the row-major block.  ds_read_b64_tr_b16 delivers exactly that: within 16 lanes, lane i passes the
//      address of 4 consecutive dims of row i/4 (dims 4 (i%4) .. +3 of a 16-dim group), and lane j receives
//      element j of rows 0..3.  Two such reads give a lane its 8 keys; their order follows the accumulator rows
//      of S^T (keys 4h .. 4h+3 and 8+4h .. 8+4h+3 of a 16-key step for lane half h), so P needs no shuffling.
#include "gemm_core.h"
#include "ssd_internal.h"

namespace ssd {

constexpr int ATT_HD = 128;
constexpr int ATT_KB = 64;                    // keys per block
constexpr int ATT_ROW_BYTES = ATT_HD * 2;     // a K or V row in LDS (unpadded)
constexpr int ATT_BLOCK_BYTES = ATT_KB * ATT_ROW_BYTES;
constexpr int ATT_O_STRIDE = ATT_HD + 8;      // output staging rows, elements
typedef short tr_v4i16 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) tr_v4i16 lds_tr_v4i16;

template <bool BF>
__global__ void __launch_bounds__(128, 2) attn_mfma_kernel(const f16_t* __restrict__ qkv, f16_t* __restrict__ out,
                                                       const AttnTile* __restrict__ tiles, int n_q_heads, int n_kv_heads) {
    __shared__ __align__(1024) unsigned char smem[2 * ATT_BLOCK_BYTES];
    unsigned char* Ks = smem;
    unsigned char* Vs = smem + ATT_BLOCK_BYTES;
    const int tid = threadIdx.x, lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int hgrp = lane / 32, lcol = lane % 32;
    // work index = tile * n_q_heads + query head, dealt so that one XCD walks a contiguous run: the heads of a KV
    // group and the tiles of an utterance (which re-read its keys and values) then share an L2
    const int work = xcd_contiguous_index(blockIdx.x, gridDim.x);
    const AttnTile t = tiles[work / n_q_heads];
    const int head = work % n_q_heads;
    const int kvh = head / (n_q_heads / n_kv_heads);
    const int d_q = n_q_heads * ATT_HD, d_kv = n_kv_heads * ATT_HD;
    const int ldq = d_q + 2 * d_kv;
    const f16_t* seq = qkv + (int64_t)t.seq_start * ldq;
    const f16_t* kbase = seq + d_q + kvh * ATT_HD;
    const __amdgpu_buffer_rsrc_t k_rsrc = make_rsrc(kbase), v_rsrc = make_rsrc(kbase + d_kv);

    const int q_first = t.q_start + wave * 32;          // first query position of this wavefront
    const int qpos = q_first + lcol;
    const bool wave_live = q_first < t.seq_len;

    // ---- global -> LDS: this wavefront fills rows 32*wave .. +31 of both blocks, instruction i rows 4i .. 4i+3;
    // a lane writes LDS chunk lane%16 of row lane/16 + 4i, which holds the logical chunk given by the swizzle.
    // Row (kb + 4i) goes into the scalar offset, so the per-lane offsets are five registers: row & 3 is that of
    // lane/16 for every i, row & 15 repeats with i % 4.
    const int ld_row = wave * 32 + lane / 16, ld_pos = lane % 16;
    const unsigned ldq2 = (unsigned)ldq * 2u;
    const unsigned v_voff = (unsigned)ld_row * ldq2 + (unsigned)(ld_pos ^ ((ld_row & 3) << 2)) * 16u;
    unsigned k_voff[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) k_voff[q] = (unsigned)ld_row * ldq2 + (unsigned)(ld_pos ^ ((ld_row + 4 * q) & 15)) * 16u;
    // Rows at and beyond seq_len are clamped to the last row (they are masked; the memory behind the last utterance
    // is not ours): only the last block of a sequence takes the per-lane route.
    auto load_block = [&](int kb, bool want_k, bool want_v) {
        if (kb + ATT_KB <= t.seq_len) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const unsigned soff = (unsigned)(kb + 4 * i) * ldq2;
                if (want_k) __builtin_amdgcn_raw_ptr_buffer_load_lds(k_rsrc, (lds_void_t*)(Ks + (wave * 8 + i) * 1024), 16, k_voff[i % 4], soff, 0, 0);
                if (want_v) __builtin_amdgcn_raw_ptr_buffer_load_lds(v_rsrc, (lds_void_t*)(Vs + (wave * 8 + i) * 1024), 16, v_voff, soff, 0, 0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int row = ld_row + 4 * i;
                const unsigned g = (unsigned)min(kb + row, t.seq_len - 1) * ldq2;
                const unsigned kc = (unsigned)(ld_pos ^ (row & 15)) * 16u;
                const unsigned vc = (unsigned)(ld_pos ^ ((row & 3) << 2)) * 16u;
                if (want_k) __builtin_amdgcn_raw_ptr_buffer_load_lds(k_rsrc, (lds_void_t*)(Ks + (wave * 8 + i) * 1024), 16, g + kc, 0, 0, 0);
                if (want_v) __builtin_amdgcn_raw_ptr_buffer_load_lds(v_rsrc, (lds_void_t*)(Vs + (wave * 8 + i) * 1024), 16, g + vc, 0, 0, 0);
            }
        }
    };
    load_block(0, true, true);                          // first, so that everything below runs under their latency

    // Q^T fragments straight into registers: lane supplies query row qpos, dims 16*kk + 8*hgrp .. +8
    f16x8_t qf[8];
    {
        const f16_t* qrow = seq + (int64_t)min(qpos, t.seq_len - 1) * ldq + head * ATT_HD + hgrp * 8;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) qf[kk] = as_f16x8(*reinterpret_cast<const uint4*>(qrow + kk * 16));
    }
    f32x16_t o_acc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float sc = 0.08838834764831845f * 1.4426950408889634f;   // log2(e) / sqrt(128)

    // ---- LDS -> fragments
    // K: row = 32*half + lcol, logical chunk 2*kk + hgrp
    int k_rd[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) k_rd[kk] = lcol * ATT_ROW_BYTES + (((2 * kk + hgrp) ^ (lcol & 15)) * 16);
    // V (transposing read): lane j of a 16-lane group passes row 4*hgrp + j/4 (+ 16 per key step, + 8 for the second
    // read) and dims 32*db + 16*(group % 2) + 4*(j % 4): chunk 4*db + 2*(group % 2) + (j % 4) / 2, half (j % 4) % 2
    int v_rd[4];
    {
        const int j = lane % 16, e = j / 4, grp2 = (lane / 16) % 2;
        const int low = 2 * grp2 + (j % 4) / 2, sub = ((j % 4) % 2) * 8;
#pragma unroll
        for (int db = 0; db < 4; ++db)
            v_rd[db] = (4 * hgrp + e) * ATT_ROW_BYTES + ((((db ^ e) << 2) | low) * 16) + sub + ATT_BLOCK_BYTES;
    }
    auto k_frag = [&](int idx) {          // idx = 8 * half + kk
        return as_f16x8(*reinterpret_cast<const uint4*>(smem + k_rd[idx % 8] + (idx / 8) * 32 * ATT_ROW_BYTES));
    };
    auto v_frag = [&](int idx) {          // idx = 4 * db + ks; key step ks covers keys 16*ks .. +15 of the block
        const unsigned char* p = smem + v_rd[idx / 4] + (idx % 4) * 16 * ATT_ROW_BYTES;
        const tr_v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_tr_v4i16*)p);
        const tr_v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_tr_v4i16*)(p + 8 * ATT_ROW_BYTES));
        typedef short v8i16 __attribute__((ext_vector_type(8)));
        const v8i16 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(f16x8_t, both);
    };

    // One barrier after the S^T products frees the K block, one after the block frees V: the next block's keys are
    // loaded under the softmax and the second product, its values under the next block's first product.
    const int kv_end = min(t.seq_len, t.q_start + 64);              // keys needed by this tile
    for (int kb = 0; kb < kv_end; kb += ATT_KB) {
        const bool active = wave_live && kb <= q_first + 31;
        const bool has_next = kb + ATT_KB < kv_end;
        f32x16_t s_acc[2];
        __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0): this wavefront's rows (and, the first time, Q) have landed
        __syncthreads();
        if (active) {
            // ---- S^T for the two 32-key halves of the block.  The K fragments are read four MFMAs ahead (a read
            // issued right before its MFMA leaves the LDS latency exposed 32 times per block).
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) s_acc[c][r] = 0.f;
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
        }
        if (has_next) {
            __syncthreads();                         // both wavefronts have read their K fragments
            load_block(kb + ATT_KB, true, false);
        }
        if (active) {
            // first V^T fragments: their latency hides behind the softmax arithmetic
            f16x8_t vq[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) vq[p] = v_frag(p);
            __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
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
            if (kb != 0) {                           // the accumulator is still zero in the first block
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o_acc[db][r] *= alpha;
            }
            // ---- O^T += V^T . P^T  (key step idx % 4 of dim block idx / 4)
#pragma unroll
            for (int idx = 0; idx < 16; ++idx) {
                o_acc[idx / 4] = mfma_32x32x16<BF>(vq[idx % 4], pf[idx % 4], o_acc[idx / 4]);
                if (idx + 4 < 16) vq[idx % 4] = v_frag(idx + 4);
            }
#pragma unroll
            for (int idx = 0; idx < 16; ++idx) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (idx + 4 < 16) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            }
        }
        __syncthreads();             // both wavefronts are done with the block's values
        if (has_next) load_block(kb + ATT_KB, false, true);
    }
    // the loop ended with a barrier: K and V are dead; the output leaves through LDS as whole 256-byte rows
    if (wave_live) {
        f16_t* wtile = reinterpret_cast<f16_t*>(smem) + wave * 32 * ATT_O_STRIDE;
        const float inv = 1.0f / l_run;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int dim = db * 32 + 8 * g + 4 * hgrp;
                uint2 w;
                w.x = op_pack2<BF>(o_acc[db][4 * g] * inv, o_acc[db][4 * g + 1] * inv);
                w.y = op_pack2<BF>(o_acc[db][4 * g + 2] * inv, o_acc[db][4 * g + 3] * inv);
                *reinterpret_cast<uint2*>(wtile + lcol * ATT_O_STRIDE + dim) = w;
            }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = q_first + i * 4 + lane / 16;
            const uint4 w = *reinterpret_cast<const uint4*>(wtile + (i * 4 + lane / 16) * ATT_O_STRIDE + (lane % 16) * 8);
            if (row < t.seq_len)
                *reinterpret_cast<uint4*>(out + (int64_t)(t.seq_start + row) * d_q + head * ATT_HD + (lane % 16) * 8) = w;
        }
    }
}

void launch_attn_mfma(const uint16_t* qkv, uint16_t* out, const AttnTile* tiles, int n_tiles, int n_q_heads,
                      int n_kv_heads, bool bf16_ops, hipStream_t st) {
    if (n_tiles <= 0) return;
    const dim3 grid(n_tiles * n_q_heads);
    if (bf16_ops) hipLaunchKernelGGL((attn_mfma_kernel<true>), grid, dim3(128), 0, st, qkv, out, tiles, n_q_heads, n_kv_heads);
    else hipLaunchKernelGGL((attn_mfma_kernel<false>), grid, dim3(128), 0, st, qkv, out, tiles, n_q_heads, n_kv_heads);
}

}  // namespace ssd
