// Fused LM head + vocabulary log-softmax + draft-token gather (the likelihoods of Eq. 5, Sec. 2.2).
//
// logits[r, v] = h_verify[r] . W_lm[v] are produced tile by tile in MFMA accumulators and reduced on
// the spot: every wavefront turns its [rows x WTN columns] slab into a partial (max, sum exp) per
// row, the lane that holds column draft_ids[r] writes that logit, and (optionally) a partial argmax
// is kept.  The full logits (rows x vocab x 4 bytes) never reach memory; what is written is
// 8 bytes per row per column group.  A second small kernel merges the partials:
//     logp[r] = logit[r, y_r] - (m + log sum_g s_g exp(m_g - m)).
#include "gemm_core16.h"
#include "ssd_internal.h"

namespace ssd {

constexpr int LM_WTN = 64;          // columns per group: every tile variant below has a 64-column wave tile

int lmhead_col_groups(int vocab) { return vocab / LM_WTN; }

template <int LM_BM, int LM_BN, int LM_WM, int LM_WN, int LM_NS, bool GREEDY, bool BF>
__global__ void __launch_bounds__(64 * LM_WM * LM_WN)
lmhead_mfma_kernel(const f16_t* __restrict__ hv, const f16_t* __restrict__ w_lm, const int32_t* __restrict__ targets,
                   int Mv, int d, int vocab, float2* __restrict__ part_ms, float* __restrict__ tgt_logit,
                   int2* __restrict__ part_arg, float descale) {
    using Tile = GemmTile<LM_BM, LM_BN, LM_WM, LM_WN, LM_NS, BF>;
    static_assert(Tile::WTN == LM_WTN, "column groups are 64 wide");
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int tiles_m = (Mv + LM_BM - 1) / LM_BM;
    // row tiles vary fastest, and the row tiles of one slab of W_lm run on one XCD (one fetch of the slab)
    const int v = xcd_contiguous_index(blockIdx.x, gridDim.x);
    const int tm = v % tiles_m, tn = v / tiles_m;
    f32x16_t acc[Tile::TM][Tile::TN];
#pragma unroll
    for (int i = 0; i < Tile::TM; ++i)
#pragma unroll
        for (int j = 0; j < Tile::TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    Tile::run(hv, w_lm, Mv, d, tm * LM_BM, tn * LM_BN, 0, d / GEMM_BK, smem_raw, acc);

    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int wm = wave / LM_WN, wn = wave % LM_WN;
    const int row0 = tm * LM_BM + wm * Tile::WTM, col0 = tn * LM_BN + wn * Tile::WTN;
    const int group = col0 / LM_WTN;
#pragma unroll
    for (int i = 0; i < Tile::TM; ++i)
#pragma unroll
        for (int j = 0; j < Tile::TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] *= descale;
    // the target ids of a block of rows first: a load inside the row loop would sit behind the stores of the
    // previous row and cost one memory round trip per row
#pragma unroll
    for (int i = 0; i < Tile::TM; ++i) {
        int tg[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) tg[r] = targets[min(row0 + acc_row(i, r, lane), Mv - 1)];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = row0 + acc_row(i, r, lane);
            const bool live = row < Mv;
            float mx = -INFINITY;
            int best_c = 0;
#pragma unroll
            for (int j = 0; j < Tile::TN; ++j) {
                const float v = acc[i][j][r];
                if (v > mx) { mx = v; best_c = col0 + acc_col(j, lane); }
            }
            const float m = row_allreduce32(mx, OpMax());
            float s = 0.f;
#pragma unroll
            for (int j = 0; j < Tile::TN; ++j) s += __expf(acc[i][j][r] - m);
            s = row_allreduce32(s, OpSum());
            if (live) {
                int tgt = tg[r];
                tgt = tgt < 0 ? 0 : (tgt >= vocab ? vocab - 1 : tgt);
                const int rel = tgt - col0 - lane % 32;
                if (rel >= 0 && rel < Tile::WTN && rel % 32 == 0) {
#pragma unroll
                    for (int j = 0; j < Tile::TN; ++j)
                        if (rel == j * 32) tgt_logit[row] = acc[i][j][r];
                }
                if (lane % 32 == 0) part_ms[(int64_t)group * Mv + row] = make_float2(m, s);
            }
            if (GREEDY) {
                // lowest column among the lanes that hold the row maximum
                int cand = (mx == m) ? best_c : 0x7fffffff;
                cand = min(cand, dpp_i<DPP_XOR1>(cand));
                cand = min(cand, dpp_i<DPP_XOR2>(cand));
                cand = min(cand, dpp_i<DPP_HALF_MIRROR>(cand));
                cand = min(cand, dpp_i<DPP_MIRROR>(cand));
                cand = min(cand, __shfl_xor(cand, 16));
                if (live && lane % 32 == 0) part_arg[(int64_t)group * Mv + row] = make_int2(__float_as_int(m), cand);
            }
        }
    }
}

// The compute-bound variant (more than 128 rows): 256 x 256 tile on v_mfma_f32_16x16x32_f16 (gemm_core16.h), and a
// reduction that needs no cross-lane steps.  A wavefront's 128 x 64 slab goes through LDS in two halves of 64
// rows, written column-major (four consecutive rows of a 16 x 16 accumulator block are one 16-byte store) with a
// column stride of 68 floats, and read back one row per lane: consecutive lanes read consecutive floats, and every
// lane scans its 64 logits in registers (maximum, lowest index of the maximum, sum of exponentials).  The
// row-wise reductions over 32 lanes of the other variants cost ten dependent cross-lane steps per row.
constexpr int LM16_COL_STRIDE = 68;                               // floats; 16-byte aligned, spreads 16 columns over all banks
constexpr int LM16_WAVE_FLOATS = 64 * LM16_COL_STRIDE;            // one half slab: 64 columns x 64 rows (+ padding)
constexpr size_t lmhead16_lds_bytes() {
    constexpr size_t ring = gemm_lds_bytes<256, 256, 2>(), stage = (size_t)8 * LM16_WAVE_FLOATS * 4;
    return ring > stage ? ring : stage;
}

template <bool BF>
__global__ void __launch_bounds__(512)
lmhead_mfma16_kernel(const f16_t* __restrict__ hv, const f16_t* __restrict__ w_lm, const int32_t* __restrict__ targets,
                     int Mv, int d, int vocab, float2* __restrict__ part_ms, float* __restrict__ tgt_logit,
                     int2* __restrict__ part_arg, float descale, int want_greedy) {
    using Tile = GemmTile16<256, 256, 2, 4, BF>;
    static_assert(Tile::WTN == LM_WTN && Tile::WTM == 128, "a wavefront owns 128 rows x one column group");
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int tiles_m = (Mv + 255) / 256;
    const int v = xcd_contiguous_index(blockIdx.x, gridDim.x);
    const int tm = v % tiles_m, tn = v / tiles_m;
    f32x4_t acc[Tile::TM][Tile::TN];
#pragma unroll
    for (int i = 0; i < Tile::TM; ++i)
#pragma unroll
        for (int j = 0; j < Tile::TN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
    Tile::run(hv, w_lm, Mv, d, tm * 256, tn * 256, 0, d / GEMM_BK, smem_raw, acc);
    // every wavefront is past the last barrier of the K loop: no fragment read is outstanding, the ring is free

    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int wm = wave / 4, wn = wave % 4;
    const int row0 = tm * 256 + wm * 128, col0 = tn * 256 + wn * 64;
    const int group = col0 / LM_WTN;
    float* T = reinterpret_cast<float*>(smem_raw) + wave * LM16_WAVE_FLOATS;
    int tgt[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int t = targets[min(row0 + 64 * h + lane, Mv - 1)];
        tgt[h] = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
    }
    const float k2 = descale * 1.4426950408889634f;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                *reinterpret_cast<f32x4_t*>(T + (16 * j + lane % 16) * LM16_COL_STRIDE + 16 * i + 4 * (lane / 16)) = acc[4 * h + i][j];
        float z[64];
#pragma unroll
        for (int c = 0; c < 64; ++c) z[c] = T[c * LM16_COL_STRIDE + lane];
        float m4[4] = {z[0], z[1], z[2], z[3]};                  // four independent chains
#pragma unroll
        for (int c = 4; c < 64; ++c) m4[c % 4] = fmaxf(m4[c % 4], z[c]);
        const float m = fmaxf(fmaxf(m4[0], m4[1]), fmaxf(m4[2], m4[3]));
        float s4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < 64; ++c) s4[c % 4] += __builtin_amdgcn_exp2f((z[c] - m) * k2);
        const float ssum = (s4[0] + s4[1]) + (s4[2] + s4[3]);
        const int row = row0 + 64 * h + lane;
        const float md = m * descale;
        const int rel = tgt[h] - col0;
        const bool has_tgt = rel >= 0 && rel < 64;
        const float zt = T[(has_tgt ? rel : 0) * LM16_COL_STRIDE + lane];
        if (row < Mv) {
            part_ms[(int64_t)group * Mv + row] = make_float2(md, ssum);
            if (has_tgt) tgt_logit[row] = zt * descale;
        }
        if (want_greedy) {
            int arg = 63;
#pragma unroll
            for (int c = 62; c >= 0; --c) arg = (z[c] == m) ? c : arg;      // lowest column that holds the maximum
            if (row < Mv) part_arg[(int64_t)group * Mv + row] = make_int2(__float_as_int(md), col0 + arg);
        }
    }
}

template <int BM, int BN, int WM, int WN, int NS, bool BF>
static void launch_lmhead_cfg(const f16_t* hv, const f16_t* w_lm, const int32_t* targets, int Mv, int d, int vocab,
                              float2* part_ms, float* tgt_logit, int2* part_arg, bool want_greedy, float descale,
                              hipStream_t st) {
    constexpr size_t lds = gemm_lds_bytes<BM, BN, NS>();
    const int tiles = ((Mv + BM - 1) / BM) * (vocab / BN);
    auto kern_greedy = lmhead_mfma_kernel<BM, BN, WM, WN, NS, true, BF>;
    auto kern_plain = lmhead_mfma_kernel<BM, BN, WM, WN, NS, false, BF>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern_greedy), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern_plain), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_set = true;
    }
    if (want_greedy)
        hipLaunchKernelGGL(kern_greedy, dim3(tiles), dim3(64 * WM * WN), lds, st, hv, w_lm, targets, Mv, d, vocab, part_ms, tgt_logit, part_arg, descale);
    else
        hipLaunchKernelGGL(kern_plain, dim3(tiles), dim3(64 * WM * WN), lds, st, hv, w_lm, targets, Mv, d, vocab, part_ms, tgt_logit, part_arg, descale);
}

// Tile by row count: up to 32 rows the whole job is streaming W_lm once (32 x 256 tile, four-stage
// ring); up to 128 rows a 128 x 64 tile; otherwise the compute-bound 256 x 256 tile (lmhead_mfma16_kernel).
template <bool BF>
static void lmhead_impl(const uint16_t* hv, const uint16_t* w_lm, const int32_t* targets, int Mv, int d, int vocab,
                        float2* part_ms, float* tgt_logit, int2* part_arg, bool want_greedy, float descale,
                        hipStream_t st) {
    if (Mv <= 32) launch_lmhead_cfg<32, 256, 1, 4, 4, BF>(hv, w_lm, targets, Mv, d, vocab, part_ms, tgt_logit, part_arg, want_greedy, descale, st);
    else if (Mv <= 128) launch_lmhead_cfg<128, 64, 4, 1, 4, BF>(hv, w_lm, targets, Mv, d, vocab, part_ms, tgt_logit, part_arg, want_greedy, descale, st);
    else {
        constexpr size_t lds = lmhead16_lds_bytes();
        static_assert(lds <= 160 * 1024, "LDS of a compute unit");
        auto kern = lmhead_mfma16_kernel<BF>;
        static bool attr_set = false;
        if (!attr_set) {
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            attr_set = true;
        }
        const int tiles = ((Mv + 255) / 256) * (vocab / 256);
        hipLaunchKernelGGL(kern, dim3(tiles), dim3(512), lds, st, (const f16_t*)hv, (const f16_t*)w_lm, targets,
                           Mv, d, vocab, part_ms, tgt_logit, part_arg, descale, want_greedy ? 1 : 0);
    }
}
void launch_lmhead_mfma(const uint16_t* hv, const uint16_t* w_lm, const int32_t* targets, int Mv, int d, int vocab,
                        float2* part_ms, float* tgt_logit, int2* part_arg, bool want_greedy, float descale,
                        bool bf16_ops, hipStream_t st) {
    if (Mv <= 0) return;
    if (bf16_ops) lmhead_impl<true>(hv, w_lm, targets, Mv, d, vocab, part_ms, tgt_logit, part_arg, want_greedy, descale, st);
    else lmhead_impl<false>(hv, w_lm, targets, Mv, d, vocab, part_ms, tgt_logit, part_arg, want_greedy, descale, st);
}

// One wavefront per row merges the per-group partials.
__global__ void __launch_bounds__(256) lmhead_finalize_kernel(const float2* __restrict__ part_ms,
                                                              const float* __restrict__ tgt_logit,
                                                              const int2* __restrict__ part_arg, int n_groups, int Mv,
                                                              float* __restrict__ logp, int32_t* __restrict__ greedy,
                                                              int32_t* __restrict__ flags) {
    const int lane = threadIdx.x % 64;
    const int row = blockIdx.x * 4 + threadIdx.x / 64;
    if (row >= Mv) return;
    float m = -INFINITY, s = 0.f;
    for (int g = lane; g < n_groups; g += 64) {
        const float2 p = part_ms[(int64_t)g * Mv + row];
        if (p.x > m) { s = s * __expf(m - p.x) + p.y; m = p.x; } else { s += p.y * __expf(p.x - m); }
    }
    const float M = group_allreduce<64>(m, OpMax());
    s = (m == -INFINITY) ? 0.f : s * __expf(m - M);
    const float S = group_allreduce<64>(s, OpSum());
    if (lane == 0) {
        const float lp = tgt_logit[row] - (M + logf(S));
        logp[row] = lp;
        if (!(fabsf(lp) < INFINITY)) raise_flag(flags, SSD_FLAG_ACT_OVERFLOW);     // non-finite likelihood: inputs were not finite
    }
    if (greedy) {
        int cand = 0x7fffffff;
        for (int g = lane; g < n_groups; g += 64) {
            const int2 a = part_arg[(int64_t)g * Mv + row];
            if (__int_as_float(a.x) == M && a.y < cand) cand = a.y;
        }
        cand = group_allreduce_i<64>(cand, OpMinI());
        if (lane == 0) greedy[row] = cand;
    }
}

void launch_lmhead_finalize(const float2* part_ms, const float* tgt_logit, const int2* part_arg, int n_groups, int Mv,
                            float* logp, int32_t* greedy, int32_t* flags, hipStream_t st) {
    if (Mv <= 0) return;
    hipLaunchKernelGGL(lmhead_finalize_kernel, dim3((Mv + 3) / 4), dim3(256), 0, st, part_ms, tgt_logit, part_arg,
                       n_groups, Mv, logp, greedy, flags);
}

}  // namespace ssd
