// CTC output layer fused with the frame statistics of the gate.
//
// The encoder's output layer (Sec. 3.1: 1024-wide states, 348 CTC symbols) produces the scores that
// Eq. 2 (greedy symbol per frame) and Eq. 3 (frame entropy) consume.  Here the scores
//     z[t, v] = enc_h[t] . W[v] + b[v]
// only ever exist in MFMA accumulators: every wavefront reduces its [rows x 64 columns] slab to
//     m = max_v z,  arg = lowest v with z = m,  S = sum_v e^(z-m),  W = sum_v e^(z-m) (z-m)
// per row (16 bytes), and a second small kernel merges the column groups of a row into
//     H_t = log S - W / S   ( = -sum_v p log p for p = softmax(z) ),   argmax_t.
// Written per frame: 16 bytes per group of 64 symbols instead of 2 x 2 bytes per symbol (a store of
// bf16 scores and the gate's load of them).  Operands are the stored bf16 values (bf16 MFMA, exact
// products, fp32 accumulation).
#include "gemm_core.h"
#include "ssd_internal.h"

namespace ssd {

constexpr int CH_WTN = 64;          // symbols per column group

template <int BM, int BN, int WM, int WN, int NS>
__global__ void __launch_bounds__(64 * WM * WN)
ctc_head_partials_kernel(const uint16_t* __restrict__ enc_h, const uint16_t* __restrict__ w_pad,
                         const float* __restrict__ bias_pad, int n_rows, int d_enc, int V, int tiles_m,
                         float4* __restrict__ part) {
    using Tile = GemmTile<BM, BN, WM, WN, NS, true>;
    static_assert(Tile::WTN == CH_WTN, "column groups are 64 wide");
    extern __shared__ __align__(16) unsigned char smem_raw[];
    // row tiles vary fastest: workgroups that run together share one slab of the (small) weight
    const int tm = blockIdx.x % tiles_m, tn = blockIdx.x / tiles_m;
    f32x16_t acc[Tile::TM][Tile::TN];
#pragma unroll
    for (int i = 0; i < Tile::TM; ++i)
#pragma unroll
        for (int j = 0; j < Tile::TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    Tile::run(reinterpret_cast<const f16_t*>(enc_h), reinterpret_cast<const f16_t*>(w_pad), n_rows, d_enc, tm * BM,
              tn * BN, 0, d_enc / GEMM_BK, smem_raw, acc);

    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int wm = wave / WN, wn = wave % WN;
    const int row0 = tm * BM + wm * Tile::WTM, col0 = tn * BN + wn * Tile::WTN;
    if (col0 >= V) return;                               // group made of padding columns only
    const int group = col0 / CH_WTN;
    float bias[Tile::TN];
    bool valid[Tile::TN];
#pragma unroll
    for (int j = 0; j < Tile::TN; ++j) {
        const int c = col0 + acc_col(j, lane);
        valid[j] = c < V;
        bias[j] = bias_pad[c];
    }
#pragma unroll
    for (int i = 0; i < Tile::TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = row0 + acc_row(i, r, lane);
            float z[Tile::TN];
            float mx = -INFINITY;
            int best_c = 0x7fffffff;
#pragma unroll
            for (int j = 0; j < Tile::TN; ++j) {
                z[j] = valid[j] ? acc[i][j][r] + bias[j] : -INFINITY;
                if (z[j] > mx) { mx = z[j]; best_c = col0 + acc_col(j, lane); }
            }
            const float m = row_allreduce32(mx, OpMax());      // finite: column col0 is valid
            const int arg = row_allmin32_i(mx == m ? best_c : 0x7fffffff);
            float s = 0.f, w = 0.f;
#pragma unroll
            for (int j = 0; j < Tile::TN; ++j) {
                const float t = z[j] - m;
                const float e = __expf(t);
                s += e;
                w += valid[j] ? e * t : 0.f;
            }
            s = row_allreduce32(s, OpSum());
            w = row_allreduce32(w, OpSum());
            if (row < n_rows && lane % 32 == 0)
                part[(int64_t)group * n_rows + row] = make_float4(m, s, w, __int_as_float(arg));
        }
}

// One thread per frame merges its column groups (coalesced: group-major partials).
__global__ void __launch_bounds__(256) ctc_head_finalize_kernel(const float4* __restrict__ part, int n_groups,
                                                                int n_rows, float* __restrict__ H,
                                                                int32_t* __restrict__ arg) {
    const int row = blockIdx.x * 256 + threadIdx.x;
    if (row >= n_rows) return;
    float M = -INFINITY;
    for (int g = 0; g < n_groups; ++g) M = fmaxf(M, part[(int64_t)g * n_rows + row].x);
    float S = 0.f, W = 0.f;
    int best = 0x7fffffff;
    for (int g = 0; g < n_groups; ++g) {
        const float4 p = part[(int64_t)g * n_rows + row];
        const float shift = p.x - M;                      // <= 0
        const float f = __expf(shift);
        S += f * p.y;
        W += f * (p.z + shift * p.y);
        if (p.x == M) best = min(best, __float_as_int(p.w));
    }
    H[row] = logf(S) - W / S;
    arg[row] = best;
}

template <int BM, int BN, int WM, int WN, int NS>
static void launch_partials(const uint16_t* enc_h, const uint16_t* w_pad, const float* bias_pad, int n_rows, int d_enc,
                            int V, int V_pad, float4* part, hipStream_t st) {
    constexpr size_t lds = gemm_lds_bytes<BM, BN, NS>();
    auto kern = ctc_head_partials_kernel<BM, BN, WM, WN, NS>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_set = true;
    }
    const int tiles_m = (n_rows + BM - 1) / BM;
    hipLaunchKernelGGL(kern, dim3(tiles_m * (V_pad / BN)), dim3(64 * WM * WN), lds, st, enc_h, w_pad, bias_pad, n_rows,
                       d_enc, V, tiles_m, part);
}

int ctc_head_groups(int V) { return (V + CH_WTN - 1) / CH_WTN; }

// enc_h [n_rows, d_enc] bf16; w_pad [V_pad, d_enc] bf16 with zero rows beyond V; bias_pad [V_pad] fp32;
// part: ctc_head_groups(V) * n_rows float4.  n_rows * d_enc * 2 must stay below 4 GiB (32-bit offsets).
void launch_ctc_head(const uint16_t* enc_h, const uint16_t* w_pad, const float* bias_pad, int n_rows, int d_enc, int V,
                     int V_pad, float4* part, float* H, int32_t* arg, hipStream_t st) {
    if (n_rows <= 0) return;
    // fewer than one 256-row tile per compute unit and column slab: halve the tile height (three LDS stages)
    if ((n_rows + 255) / 256 < 256) launch_partials<128, 256, 2, 4, 3>(enc_h, w_pad, bias_pad, n_rows, d_enc, V, V_pad, part, st);
    else launch_partials<256, 256, 2, 4, 2>(enc_h, w_pad, bias_pad, n_rows, d_enc, V, V_pad, part, st);
    hipLaunchKernelGGL(ctc_head_finalize_kernel, dim3((n_rows + 255) / 256), dim3(256), 0, st, part, ctc_head_groups(V),
                       n_rows, H, arg);
}

// zero-padded copy of the output layer: rows [V, V_pad) are zero, bias there is zero too (masked by column index)
__global__ void ctc_head_pack_kernel(const uint16_t* __restrict__ w, const float* __restrict__ bias, int V, int V_pad,
                                     int d_enc, uint16_t* __restrict__ w_pad, float* __restrict__ bias_pad) {
    const int64_t n = (int64_t)V_pad * d_enc;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        w_pad[i] = (i / d_enc < V) ? w[i] : (uint16_t)0;
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c < V_pad) bias_pad[c] = (c < V && bias) ? bias[c] : 0.f;
}

void launch_ctc_head_pack(const uint16_t* w, const float* bias, int V, int V_pad, int d_enc, uint16_t* w_pad,
                          float* bias_pad, hipStream_t st) {
    const int64_t n = (int64_t)V_pad * d_enc;
    const unsigned grid = (unsigned)std::max<int64_t>((V_pad + 255) / 256, std::min<int64_t>((n + 255) / 256, 4096));
    hipLaunchKernelGGL(ctc_head_pack_kernel, dim3(grid), dim3(256), 0, st, w, bias, V, V_pad, d_enc, w_pad, bias_pad);
}

}  // namespace ssd
