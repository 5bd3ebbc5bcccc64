// Internal declarations shared by the kernel files and the C-ABI layer.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/ssd.h"

namespace ssd {

// ---- gate.hip
void launch_gate(const void* logits, int dtype, int64_t n_rows, int V, const int32_t* cu_frames_dev, int B,
                 int blank, float tau, float* H, int32_t* arg, float* max_entropy, uint8_t* gate_pass,
                 int32_t* draft, int32_t* draft_len, hipStream_t st);

// second half of the gate on its own: per-utterance max entropy, threshold test and collapse
// (frame ranges are clamped into [0, n_rows] on the device)
void launch_gate_utterances(const float* H, const int32_t* arg, const int32_t* cu_frames_dev, int64_t n_rows, int B, int blank,
                            float tau, float* max_entropy, uint8_t* gate_pass, int32_t* draft, int32_t* draft_len,
                            hipStream_t st);

// ---- ctc_head.hip: output layer of the CTC encoder fused with the frame statistics of the gate
int ctc_head_groups(int V);      // groups of 64 symbols that hold at least one real symbol
int ctc_head_padded(int V);      // symbol count after padding
void launch_ctc_head_pack(const uint16_t* w, const float* bias, int V, int V_pad, int d_enc, uint16_t* w_pad,
                          float* bias_pad, hipStream_t st);
// part: ctc_head_groups(V) * n_rows float4 of scratch; n_rows * d_enc * 2 bytes must stay below 4 GiB
void launch_ctc_head(const uint16_t* enc_h, const uint16_t* w_pad, const float* bias_pad, int n_rows, int d_enc, int V,
                     int V_pad, float4* part, float* H, int32_t* arg, hipStream_t st);

// ---- qformer.hip: windowed cross-attention of the projector (Sec. 3.1)
constexpr int QF_SCORE_COLS = 64;    // columns of the fused weight that hold the folded (query, head) score rows
constexpr int QF_MAX_WINDOW = 32;
constexpr int QF_MAX_QUERIES = 4;
struct QWindow { int32_t frame0, n_frames; };
int qformer_cat_rows(int d_h);       // rows of the fused [scores | values] weight, padded to a multiple of 256
// w_cat [qformer_cat_rows(d_h), d_enc] bf16: rows j * n_heads + h hold w_k[head h]^T q_proj[j, head h] / sqrt(d_head),
// rows 64 .. 64 + d_h - 1 hold w_v, the rest is zero
void launch_qformer_fold(const uint16_t* q_proj, const uint16_t* w_k, const uint16_t* w_v, int n_q, int n_heads, int d_h,
                         int d_enc, uint16_t* w_cat, hipStream_t st);
// scores [frames, 64] fp32 and vals [frames, d_h] IEEE half = enc_h w_cat^T; for every window: softmax of its score
// columns over its frames, then the weighted sum of its value columns: o [n_windows * n_q, d_h] bf16
void launch_qformer_pool(const float* scores, const uint16_t* vals, const QWindow* wins, int n_windows, int n_q, int n_heads,
                         int d_h, uint16_t* o, hipStream_t st);

// ---- row metadata built on the host for one verify_forward call
// src code of a decoder row: speech rows hold the speech_emb row index; token rows hold
// SRC_PROMPT | index into prompt_ids or SRC_DRAFT | index into draft_ids.
constexpr int32_t SRC_PROMPT = 0x40000000;
constexpr int32_t SRC_DRAFT = (int32_t)0x80000000u;
constexpr int32_t SRC_MASK = 0x3fffffff;

// One attention work item: a tile of query rows of one utterance.
struct AttnTile {
    int32_t seq_start;   // first decoder row of the utterance
    int32_t seq_len;     // rows in the utterance
    int32_t q_start;     // first query position of this tile (multiple of the tile height)
    int32_t pad;
};

// ---- elementwise.hip
// flags (may be NULL): SSD_FLAG_TOKEN_CLAMPED is raised if a token id had to be clamped into [0, vocab)
void launch_embed_rows(int dtype, const void* speech_emb, const void* embed, const int32_t* prompt_ids,
                       const int32_t* draft_ids, const int32_t* row_src, int M, int d, int vocab, float* x,
                       int32_t* flags, hipStream_t st);
void launch_gather_rows(const void* src, const int32_t* row_idx, int n_rows, int64_t row_bytes, void* dst, hipStream_t st);
// out[i] = src[idx[i]], passed through table (clamped into [0, n_table)) when table is not NULL
void launch_gather_ids(const int32_t* src, const int32_t* idx, int n, const int32_t* table, int n_table, int32_t* out, hipStream_t st);
// a = rmsnorm(x) * gain;  rows optionally gathered through row_idx (NULL = identity).
// If n_splits > 1, x[row] is first increased by partials[s][row] for s = 0..n_splits-1 (fixed order;
// partials is [n_splits][M][d] fp32) and, when row_idx is NULL, written back.
// flags (may be NULL): SSD_FLAG_ACT_OVERFLOW is raised when a half-precision output had to be saturated
void launch_rmsnorm(int dtype, float* x, const void* gain, const int32_t* row_idx, int n_rows, int d,
                    float eps, void* out, const float* partials, int n_splits, int64_t split_stride, int32_t* flags,
                    bool bf16_ops, hipStream_t st);

// ---- f32_path.hip (all-fp32 decoder for the tiny configuration)
enum F32Epilogue { F32_STORE = 0, F32_ADD = 1 };
void launch_gemm_f32(const float* A, const float* W, float* C, int M, int N, int K, int epilogue, hipStream_t st);
void launch_rope_f32(float* qkv, const int32_t* pos, const float* rope_tab, int M, int n_heads_rot, int head_dim,
                     int row_stride, hipStream_t st);
void launch_swiglu_f32(const float* gu, float* h, int M, int d_ff, hipStream_t st);
void launch_attn_f32(const float* qkv, float* out, const AttnTile* tiles, int n_tiles, int n_q_heads,
                     int n_kv_heads, int head_dim, hipStream_t st);
void launch_lmhead_f32(const float* hv, const float* w_lm, const int32_t* targets, int Mv, int d, int vocab,
                       float* logp, int32_t* greedy, hipStream_t st);

// ---- gemm_mfma.hip (16-bit MFMA GEMMs with fused epilogues), attn_mfma.hip, lmhead_mfma.hip.
// Activations and converted weights are 16-bit operand patterns: IEEE half, or bfloat16 when bf16_ops is set (the
// context's operand type); `descale` undoes the weight scale (1 for bfloat16 operands).
// row_slot / kc / vc (all or none): rows with row_slot[row] >= 0 also store their rotated k part and their v
// part into the K/V cache of this layer at that slot (what launch_kv_store does as a separate pass)
// W_stream (may be NULL): the same weights in the stream layout of launch_stream_layout, read when at
// most 32 rows are projected
// rope_rows (may be NULL): rope_tab[pos[row]] gathered per row, [M][64] (cos, sin); read instead of pos and rope_tab
void launch_gemm_qkv_rope(const uint16_t* A, const uint16_t* Wqkv_packed, const void* W_stream, uint16_t* qkv, const int32_t* pos,
                          const float* rope_tab, int M, int d_model, int d_q, int d_kv, float descale,
                          const int32_t* row_slot, uint16_t* kc, uint16_t* vc, const float* rope_rows, int32_t* flags,
                          bool bf16_ops, hipStream_t st);
constexpr int SKINNY_MAX_ROWS = 128;     // at most this many decoder rows: weight-streaming GEMM variants
constexpr int SKINNY_MAX_SPLITS = 8;
int gemm_residual_splits(int M, int N, int K, bool have_stream);
// returns the number of K splits written to `partials` ([splits][M][N] fp32), or 1 if x was updated in place
int launch_gemm_residual(const uint16_t* A, const uint16_t* W, const void* W_stream, float* x, float* partials, int M, int N, int K,
                         float descale, bool bf16_ops, hipStream_t st);
void launch_gemm_swiglu(const uint16_t* A, const uint16_t* Wgu_packed, const void* W_stream, uint16_t* h, int M, int d_ff, int K,
                        float descale, int32_t* flags, bool bf16_ops, hipStream_t st);
// plain products C[M,N] = A[M,K] W[N,K]^T with fp32 accumulation, stored as fp32 or rounded to the operand type
// (N % 256 == 0, K % 64 == 0, row-major 16-bit operands of the type bf16_ops selects)
// C = A W^T with W = [64 score rows | d_h value rows | zero rows up to N]: scores [M, 64] fp32, vals [M, d_h] IEEE half (saturating)
void launch_gemm_scores_values(const uint16_t* A, const uint16_t* W, float* scores, uint16_t* vals, int M, int N, int K, int d_h,
                               int32_t* flags, bool bf16_ops, hipStream_t st);
void launch_gemm_store_16(const uint16_t* A, const uint16_t* W, uint16_t* C, int M, int N, int K, bool bf16_ops, hipStream_t st);
// second copy of an f16 weight matrix W[N,K] for the few-row kernel (N % 64 == 0, K % 256 == 0)
bool stream_layout_supported(int N, int K);
void launch_stream_layout(const uint16_t* w, void* out, int N, int K, hipStream_t st);
void launch_attn_mfma(const uint16_t* qkv, uint16_t* out, const AttnTile* tiles, int n_tiles, int n_q_heads,
                      int n_kv_heads, bool bf16_ops, hipStream_t st);
// partial log-sum-exp of the LM head over column groups; see lmhead_mfma.hip
int lmhead_col_groups(int vocab);
void launch_lmhead_mfma(const uint16_t* hv, const uint16_t* w_lm, const int32_t* targets, int Mv, int d,
                        int vocab, float2* part_ms, float* tgt_logit, int2* part_arg, bool want_greedy,
                        float descale, bool bf16_ops, hipStream_t st);
// flags (may be NULL): SSD_FLAG_ACT_OVERFLOW is raised when a log-likelihood is not finite
void launch_lmhead_finalize(const float2* part_ms, const float* tgt_logit, const int2* part_arg, int n_groups,
                            int Mv, float* logp, int32_t* greedy, int32_t* flags, hipStream_t st);

// weight re-layout at context creation
// (bf16 weights are converted to f16 times the power of two `scale`, or kept as they are when scale is 0;
// fp32 weights are copied)
void launch_absmax(int dtype, const void* w, int64_t n, unsigned int* out_bits, hipStream_t st);
// inexact (device counter, may be NULL) is increased by the number of values whose half representation is not exact
void launch_convert_weight(int dtype, const void* w, void* out, int rows, int cols, float scale, unsigned long long* inexact,
                           hipStream_t st);
void launch_pack_qkv(int dtype, const void* wq, const void* wk, const void* wv, void* out, int d_q, int d_kv,
                     int d_model, int head_dim, float scale, unsigned long long* inexact, hipStream_t st);
void launch_pack_gate_up(int dtype, const void* wg, const void* wu, void* out, int d_ff, int d_model, float scale,
                         unsigned long long* inexact, hipStream_t st);

// ---- ar_decode.hip (auto-regressive fallback): K/V cache of one layer is K [slots, d_kv], V [slots, d_kv]
// in the activation type (IEEE half for bf16-stored models, fp32 otherwise); row_slot < 0 skips a row
void launch_kv_store(int dtype, const void* qkv, const int32_t* row_slot, int n_rows, int d_q, int d_kv, void* kc,
                     void* vc, hipStream_t st);
void launch_decode_attn(int dtype, const void* qkv, const void* kc, const void* vc, const int32_t* kv_start,
                        const int32_t* n_ctx, int Br, int n_q_heads, int n_kv_heads, int head_dim, void* out,
                        bool bf16_ops, hipStream_t st);

// head_dim 128, half precision: decode attention that finishes the QKV projection itself.  qkv_part is
// [n_splits][Br][d_q + 2 d_kv] fp32 partial sums in the packed column order of the fused QKV weight; the
// kernel adds the splits, rotates q and k at position n_ctx[b] - 1 (the number of rows the utterance already
// has in the cache), stores the new k / v row at cache slot kv_start[b] + n_ctx[b] - 1 and attends to the
// cached rows plus the new one.
void launch_decode_attn_fused(const float* qkv_part, int n_splits, const float* rope_tab, void* kc, void* vc,
                              const int32_t* kv_start, const int32_t* n_ctx, int Br, int n_q_heads, int n_kv_heads,
                              void* out, int32_t* flags, bool bf16_ops, hipStream_t st);
// QKV projection left as K-split partial sums for launch_decode_attn_fused; returns the split count, or 0 if
// the shape is not served (then nothing was launched)
int launch_gemm_qkv_partial(const uint16_t* A, const void* W_stream, float* part, int M, int d_model, int N, float descale,
                            bool bf16_ops, hipStream_t st);

// threshold grids: outputs are [n_tau][B] / [n_tau][Bv]
void launch_gate_grid(const float* max_entropy, int B, const float* taus_dev, int n_tau, uint8_t* gate_pass, hipStream_t st);
void launch_accept_grid(const float* logp, const int32_t* cu_draft_dev, int Bv, const float* ln_taus_dev, int n_tau,
                        int32_t* accept_len, uint8_t* all_accepted, hipStream_t st);

// measurement aid: MFMA-only loop (sink: n_workgroups*512 floats, clocks: 2 x int64)
// measurement aid: plain streaming read of `bytes` (multiple of 16) from buf
void launch_hbm_read(const void* buf, size_t bytes, uint32_t* sink, hipStream_t st);
void launch_mfma_ceiling(float* sink, long long* clocks, int n_workgroups, int iters, hipStream_t st);

// ---- accept (shared by both dtypes): first failing token per utterance
void launch_accept_scan(const float* logp, const int32_t* cu_draft_dev, int Bv, float ln_tau, int32_t* accept_len,
                        uint8_t* all_accepted, hipStream_t st);

}  // namespace ssd
