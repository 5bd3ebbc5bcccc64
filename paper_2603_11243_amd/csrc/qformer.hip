// Windowed cross-attention of the query-transformer projector (Sec. 3.1): every window of 15 consecutive encoder
// frames is summarised by 3 trainable queries, which turns the frame sequence into the 5 times shorter sequence
// of acoustic embeddings that the LLM is conditioned on (the g of Sec. 2.2).
//
// The queries are constants of the model, so the score of frame t for (query j, head h),
//     q_proj[j, h] . (w_k h_t)[h] / sqrt(d_head)  =  (w_k[h]^T q_proj[j, h] / sqrt(d_head)) . h_t,
// is a fixed linear function of the frame: the key projection folds into n_q * n_heads score rows.  Those rows and
// w_v form one weight matrix, and the path is
//   1. [scores | values] = enc_h w_cat^T                  one MFMA GEMM (gemm_mfma.hip): scores [frames, 64] fp32,
//                                                         values [frames, d_h] IEEE half
//   2. per window: softmax over its frames of each score column, weighted sum of the value columns   (here)
//   3. g [3 windows, d_out] = o w_o^T                      one MFMA GEMM, stored in the storage type of speech_emb
// Windows never cross an utterance; the last window of an utterance may hold fewer frames.
#include "device_utils.h"
#include "ssd_internal.h"

namespace ssd {

int qformer_cat_rows(int d_h) { return (QF_SCORE_COLS + d_h + 255) / 256 * 256; }

// One workgroup per row of w_cat.
__global__ void __launch_bounds__(256) qformer_fold_kernel(const bf16_t* __restrict__ q_proj, const bf16_t* __restrict__ w_k,
                                                           const bf16_t* __restrict__ w_v, int n_q, int n_heads, int d_h,
                                                           int d_enc, bf16_t* __restrict__ w_cat) {
    const int r = blockIdx.x;
    bf16_t* dst = w_cat + (int64_t)r * d_enc;
    if (r < n_q * n_heads) {
        const int j = r / n_heads, h = r % n_heads, dh = d_h / n_heads;
        const float scale = 1.0f / sqrtf((float)dh);
        for (int e = threadIdx.x; e < d_enc; e += 256) {
            float acc = 0.f;
            for (int c = 0; c < dh; ++c)
                acc = fmaf(bf16_to_f32(q_proj[j * d_h + h * dh + c]), bf16_to_f32(w_k[(int64_t)(h * dh + c) * d_enc + e]), acc);
            dst[e] = f32_to_bf16(acc * scale);
        }
    } else if (r >= QF_SCORE_COLS && r < QF_SCORE_COLS + d_h) {
        const bf16_t* src = w_v + (int64_t)(r - QF_SCORE_COLS) * d_enc;
        for (int e = threadIdx.x; e < d_enc; e += 256) dst[e] = src[e];
    } else {
        for (int e = threadIdx.x; e < d_enc; e += 256) dst[e] = 0;
    }
}

void launch_qformer_fold(const uint16_t* q_proj, const uint16_t* w_k, const uint16_t* w_v, int n_q, int n_heads, int d_h,
                         int d_enc, uint16_t* w_cat, hipStream_t st) {
    hipLaunchKernelGGL(qformer_fold_kernel, dim3(qformer_cat_rows(d_h)), dim3(256), 0, st, q_proj, w_k, w_v, n_q, n_heads, d_h,
                       d_enc, w_cat);
}

// One workgroup per window.  Scores of the window's frames go through LDS, one thread normalises one
// (query, head) column over the frames, then every thread owns four consecutive value columns (one 8-byte load
// per frame, whole rows coalesced) and accumulates their n_q weighted sums over the frames.
template <int NQ>
__global__ void __launch_bounds__(256) qformer_pool_kernel(const float* __restrict__ scores, const f16_t* __restrict__ vals,
                                                           const QWindow* __restrict__ wins, int n_heads, int d_h,
                                                           bf16_t* __restrict__ o) {
    __shared__ float p_s[QF_SCORE_COLS][QF_MAX_WINDOW + 1];
    const QWindow w = wins[blockIdx.x];
    const int n_pairs = NQ * n_heads;
    const float* sbase = scores + (int64_t)w.frame0 * QF_SCORE_COLS;
    for (int i = threadIdx.x; i < w.n_frames * QF_SCORE_COLS; i += 256)        // the window's scores are one contiguous piece
        p_s[i % QF_SCORE_COLS][i / QF_SCORE_COLS] = sbase[i];
    __syncthreads();
    if ((int)threadIdx.x < n_pairs) {
        float* p = p_s[threadIdx.x];
        float m = -INFINITY;
        for (int t = 0; t < w.n_frames; ++t) m = fmaxf(m, p[t]);
        float sum = 0.f;
        for (int t = 0; t < w.n_frames; ++t) { const float e = __expf(p[t] - m); p[t] = e; sum += e; }
        const float inv = 1.0f / sum;
        for (int t = 0; t < w.n_frames; ++t) p[t] *= inv;
    }
    __syncthreads();
    const int dh = d_h / n_heads;                                              // a multiple of 4: four columns share a head
    const f16_t* vbase = vals + (int64_t)w.frame0 * d_h;
    for (int c = 4 * threadIdx.x; c < d_h; c += 1024) {
        const int h = c / dh;
        float acc[NQ][4];
#pragma unroll
        for (int j = 0; j < NQ; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[j][e] = 0.f;
        for (int t = 0; t < w.n_frames; ++t) {
            const uint2 raw = *reinterpret_cast<const uint2*>(vbase + (int64_t)t * d_h + c);
            const float v[4] = {f16_to_f32((f16_t)(raw.x & 0xffffu)), f16_to_f32((f16_t)(raw.x >> 16)),
                                f16_to_f32((f16_t)(raw.y & 0xffffu)), f16_to_f32((f16_t)(raw.y >> 16))};
#pragma unroll
            for (int j = 0; j < NQ; ++j) {
                const float p = p_s[j * n_heads + h][t];
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[j][e] = fmaf(p, v[e], acc[j][e]);
            }
        }
#pragma unroll
        for (int j = 0; j < NQ; ++j)
            *reinterpret_cast<uint2*>(o + ((int64_t)blockIdx.x * NQ + j) * d_h + c) =
                make_uint2(pack_bf16x2(acc[j][0], acc[j][1]), pack_bf16x2(acc[j][2], acc[j][3]));
    }
}

void launch_qformer_pool(const float* scores, const uint16_t* vals, const QWindow* wins, int n_windows, int n_q, int n_heads,
                         int d_h, uint16_t* o, hipStream_t st) {
    if (n_windows <= 0) return;
#define SSD_QF(NQ) hipLaunchKernelGGL(qformer_pool_kernel<NQ>, dim3(n_windows), dim3(256), 0, st, scores, vals, wins, n_heads, d_h, o)
    if (n_q == 1) SSD_QF(1); else if (n_q == 2) SSD_QF(2); else if (n_q == 3) SSD_QF(3); else SSD_QF(4);
#undef SSD_QF
}

}  // namespace ssd
