// CTC output layer fused with the frame statistics of the gate.
//
// The encoder's output layer (Sec. 3.1: 1024-wide states, 348 CTC symbols) produces the scores that
// Eq. 2 (greedy symbol per frame) and Eq. 3 (frame entropy) consume.  Here the scores
//     z[t, v] = enc_h[t] . W[v] + b[v]
// only ever exist in MFMA accumulators.  The product is formed transposed, Z^T = W . enc_h^T, so that
// an accumulator lane owns one frame (its column) and 16 symbols per 32x32 block (its registers):
// the per-frame reductions over symbols run inside the lane, with a single exchange between the two
// lane halves at the end.  Every wavefront reduces its [64 symbols x frames] slab to
//     m = max_v z,  arg = lowest v with z = m,  S = sum_v e^(z-m),  W = sum_v e^(z-m) (z-m)
// per frame (16 bytes), and a second small kernel merges the symbol groups of a frame into
//     H_t = log S - W / S   ( = -sum_v p log p for p = softmax(z) ),   argmax_t.
// Written per frame: 16 bytes per group of 64 symbols instead of 2 x 2 bytes per symbol (a store of
// bf16 scores and the gate's load of them).  Operands are the stored bf16 values (bf16 MFMA, exact
// products, fp32 accumulation); the accumulators start at the bias, and symbols added as padding
// have zero weights and bias -inf, i.e. probability zero.
#include "gemm_core.h"
#include "ssd_internal.h"

namespace ssd {

constexpr int CH_BM = 128;          // symbols per tile
constexpr int CH_GROUP = 64;        // symbols per partial: the wave tile height of every variant below
constexpr int CH_PAD = 128;         // symbol count is padded to a multiple of this

template <int BN, int WM, int WN, int NS>
__global__ void __launch_bounds__(64 * WM * WN)
ctc_head_partials_kernel(const uint16_t* __restrict__ enc_h, const uint16_t* __restrict__ w_pad,
                         const float* __restrict__ bias_pad, int n_rows, int d_enc, int V, int V_pad,
                         float4* __restrict__ part) {
    using Tile = GemmTile<CH_BM, BN, WM, WN, NS, true>;
    static_assert(Tile::WTM == CH_GROUP, "one partial per wave tile of 64 symbols");
    extern __shared__ __align__(16) unsigned char smem_raw[];
    // symbol tiles vary fastest, and the tiles of one slab of frames run on one XCD (one fetch of the slab)
    const int tiles_v = V_pad / CH_BM;
    const int v = xcd_contiguous_index(blockIdx.x, gridDim.x);
    const int tv = v % tiles_v, tf = v / tiles_v;
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int wm = wave / WN, wn = wave % WN;
    const int sym0 = tv * CH_BM + wm * Tile::WTM;            // first symbol of this wavefront
    const int frame0 = tf * BN + wn * Tile::WTN;
    const int half = lane / 32;

    f32x16_t acc[Tile::TM][Tile::TN];
#pragma unroll
    for (int i = 0; i < Tile::TM; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 b4 = *reinterpret_cast<const float4*>(bias_pad + sym0 + i * 32 + 8 * q + 4 * half);
#pragma unroll
            for (int j = 0; j < Tile::TN; ++j) {
                acc[i][j][4 * q + 0] = b4.x; acc[i][j][4 * q + 1] = b4.y;
                acc[i][j][4 * q + 2] = b4.z; acc[i][j][4 * q + 3] = b4.w;
            }
        }
    Tile::run(reinterpret_cast<const f16_t*>(w_pad), reinterpret_cast<const f16_t*>(enc_h), V_pad, d_enc, tv * CH_BM,
              tf * BN, 0, d_enc / GEMM_BK, smem_raw, acc, n_rows);

    if (sym0 >= V) return;                                   // slab made of padding symbols only
    const int group = sym0 / CH_GROUP;
    constexpr float LOG2E = 1.4426950408889634f;
#pragma unroll
    for (int j = 0; j < Tile::TN; ++j) {
        const int frame = frame0 + j * 32 + lane % 32;
        float m = -INFINITY;
#pragma unroll
        for (int i = 0; i < Tile::TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; r += 2) m = fmaxf(m, fmaxf(acc[i][j][r], acc[i][j][r + 1]));
        m = fmaxf(m, __shfl_xor(m, 32));                     // finite: symbol sym0 is real
        const float mL = m * LOG2E;
        float s = 0.f, w = 0.f;
        int rel = 0x7fffffff;                                // symbol index relative to sym0 + 4*half
        // descending symbol order: the last match is the lowest index
#pragma unroll
        for (int i = Tile::TM - 1; i >= 0; --i)
#pragma unroll
            for (int r = 15; r >= 0; --r) {
                const float z = acc[i][j][r];
                const float t2 = fmaf(z, LOG2E, -mL);        // (z - m) log2 e  <= 0; -inf for padding
                const float e = __builtin_amdgcn_exp2f(t2);
                s += e;
                w = fmaf(e, fmaxf(t2, -200.f), w);           // e is 0 there; keeps 0 * inf out
                if (z == m) rel = i * 32 + 8 * (r / 4) + (r % 4);
            }
        int arg = rel == 0x7fffffff ? rel : sym0 + 4 * half + rel;
        s += __shfl_xor(s, 32);
        w += __shfl_xor(w, 32);
        arg = min(arg, __shfl_xor(arg, 32));
        if (frame < n_rows && half == 0)
            part[(int64_t)group * n_rows + frame] = make_float4(m, s, w * (1.0f / LOG2E), __int_as_float(arg));
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

template <int BN, int WM, int WN, int NS>
static void launch_partials(const uint16_t* enc_h, const uint16_t* w_pad, const float* bias_pad, int n_rows, int d_enc,
                            int V, int V_pad, float4* part, hipStream_t st) {
    constexpr size_t lds = gemm_lds_bytes<CH_BM, BN, NS>();
    auto kern = ctc_head_partials_kernel<BN, WM, WN, NS>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_set = true;
    }
    const int tiles_f = (n_rows + BN - 1) / BN;
    hipLaunchKernelGGL(kern, dim3(tiles_f * (V_pad / CH_BM)), dim3(64 * WM * WN), lds, st, enc_h, w_pad, bias_pad,
                       n_rows, d_enc, V, V_pad, part);
}

int ctc_head_groups(int V) { return (V + CH_GROUP - 1) / CH_GROUP; }
int ctc_head_padded(int V) { return (V + CH_PAD - 1) / CH_PAD * CH_PAD; }

// enc_h [n_rows, d_enc] bf16; w_pad [V_pad, d_enc] bf16 with zero rows beyond V; bias_pad [V_pad] fp32, -inf
// beyond V; part: ctc_head_groups(V) * n_rows float4.  n_rows * d_enc * 2 must stay below 4 GiB.
void launch_ctc_head(const uint16_t* enc_h, const uint16_t* w_pad, const float* bias_pad, int n_rows, int d_enc, int V,
                     int V_pad, float4* part, float* H, int32_t* arg, hipStream_t st) {
    if (n_rows <= 0) return;
    launch_partials<256, 2, 4, 3>(enc_h, w_pad, bias_pad, n_rows, d_enc, V, V_pad, part, st);
    hipLaunchKernelGGL(ctc_head_finalize_kernel, dim3((n_rows + 255) / 256), dim3(256), 0, st, part, ctc_head_groups(V),
                       n_rows, H, arg);
}

// padded copy of the output layer: rows [V, V_pad) are zero and their bias is -inf
__global__ void ctc_head_pack_kernel(const uint16_t* __restrict__ w, const float* __restrict__ bias, int V, int V_pad,
                                     int d_enc, uint16_t* __restrict__ w_pad, float* __restrict__ bias_pad) {
    const int64_t n = (int64_t)V_pad * d_enc;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        w_pad[i] = (i / d_enc < V) ? w[i] : (uint16_t)0;
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c < V_pad) bias_pad[c] = c < V ? (bias ? bias[c] : 0.f) : -INFINITY;
}

void launch_ctc_head_pack(const uint16_t* w, const float* bias, int V, int V_pad, int d_enc, uint16_t* w_pad,
                          float* bias_pad, hipStream_t st) {
    const int64_t n = (int64_t)V_pad * d_enc;
    const unsigned grid = (unsigned)std::max<int64_t>((V_pad + 255) / 256, std::min<int64_t>((n + 255) / 256, 4096));
    hipLaunchKernelGGL(ctc_head_pack_kernel, dim3(grid), dim3(256), 0, st, w, bias, V, V_pad, d_enc, w_pad, bias_pad);
}

}  // namespace ssd
