// Fused LM head + vocabulary log-softmax + draft-token gather (the likelihoods of Eq. 5, Sec. 2.2).
//
// logits[r, v] = h_verify[r] . W_lm[v] are produced tile by tile in MFMA accumulators and reduced on
// the spot: every wavefront turns its [rows x WTN columns] slab into a partial (max, sum exp) per
// row, the lane that holds column draft_ids[r] writes that logit, and (optionally) a partial argmax
// is kept.  The full logits (rows x vocab x 4 bytes) never reach memory; what is written is
// 8 bytes per row per column group.  A second small kernel merges the partials:
//     logp[r] = logit[r, y_r] - (m + log sum_g s_g exp(m_g - m)).
#include "gemm_core.h"
#include "ssd_internal.h"

namespace ssd {

constexpr int LM_WTN = 64;          // columns per group: every tile variant below has a 64-column wave tile

int lmhead_col_groups(int vocab) { return vocab / LM_WTN; }

template <int LM_BM, int LM_BN, int LM_WM, int LM_WN, int LM_NS, bool GREEDY>
__global__ void __launch_bounds__(64 * LM_WM * LM_WN)
lmhead_mfma_kernel(const f16_t* __restrict__ hv, const f16_t* __restrict__ w_lm, const int32_t* __restrict__ targets,
                   int Mv, int d, int vocab, float2* __restrict__ part_ms, float* __restrict__ tgt_logit,
                   int2* __restrict__ part_arg, float descale) {
    using Tile = GemmTile<LM_BM, LM_BN, LM_WM, LM_WN, LM_NS>;
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

template <int BM, int BN, int WM, int WN, int NS>
static void launch_lmhead_cfg(const f16_t* hv, const f16_t* w_lm, const int32_t* targets, int Mv, int d, int vocab,
                              float2* part_ms, float* tgt_logit, int2* part_arg, bool want_greedy, float descale,
                              hipStream_t st) {
    constexpr size_t lds = gemm_lds_bytes<BM, BN, NS>();
    const int tiles = ((Mv + BM - 1) / BM) * (vocab / BN);
    auto kern_greedy = lmhead_mfma_kernel<BM, BN, WM, WN, NS, true>;
    auto kern_plain = lmhead_mfma_kernel<BM, BN, WM, WN, NS, false>;
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
// ring); up to 128 rows a 128 x 64 tile; otherwise the compute-bound 256 x 256 tile.
void launch_lmhead_mfma(const uint16_t* hv, const uint16_t* w_lm, const int32_t* targets, int Mv, int d, int vocab,
                        float2* part_ms, float* tgt_logit, int2* part_arg, bool want_greedy, float descale,
                        hipStream_t st) {
    if (Mv <= 0) return;
    if (Mv <= 32) launch_lmhead_cfg<32, 256, 1, 4, 4>(hv, w_lm, targets, Mv, d, vocab, part_ms, tgt_logit, part_arg, want_greedy, descale, st);
    else if (Mv <= 128) launch_lmhead_cfg<128, 64, 4, 1, 4>(hv, w_lm, targets, Mv, d, vocab, part_ms, tgt_logit, part_arg, want_greedy, descale, st);
    else launch_lmhead_cfg<256, 256, 2, 4, 2>(hv, w_lm, targets, Mv, d, vocab, part_ms, tgt_logit, part_arg, want_greedy, descale, st);
}

// One wavefront per row merges the per-group partials.
__global__ void __launch_bounds__(256) lmhead_finalize_kernel(const float2* __restrict__ part_ms,
                                                              const float* __restrict__ tgt_logit,
                                                              const int2* __restrict__ part_arg, int n_groups, int Mv,
                                                              float* __restrict__ logp, int32_t* __restrict__ greedy) {
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
    if (lane == 0) logp[row] = tgt_logit[row] - (M + logf(S));
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
                            float* logp, int32_t* greedy, hipStream_t st) {
    if (Mv <= 0) return;
    hipLaunchKernelGGL(lmhead_finalize_kernel, dim3((Mv + 3) / 4), dim3(256), 0, st, part_ms, tgt_logit, part_arg,
                       n_groups, Mv, logp, greedy);
}

}  // namespace ssd
