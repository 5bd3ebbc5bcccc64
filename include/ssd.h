/*
 * ssd.h -- C ABI of the gate -> verify -> accept hot path of CTC-draft self-speculative
 * decoding for speech-aware LLMs, hand-written for AMD gfx950 (MI355X).
 *
 * The three compute calls follow the paper's statement of the method:
 *   ctc_gate        Sec. 2.1: greedy CTC path (Eq. 2), collapse map B, frame-entropy gate (Eq. 3)
 *   verify_forward  Sec. 2.2: one causal decoder forward over [speech emb g; prompt; draft] (Eq. 4)
 *   accept_prefix   Sec. 2.2-2.3: draft-token log-likelihoods, relaxed acceptance (Eq. 5) and the
 *                   longest verified prefix that auto-regressive fallback resumes from (Eq. 7)
 *
 * Conventions
 *   - "dev" pointers are device (HBM) pointers owned by the caller; "host" pointers are ordinary
 *     host memory.  The library keeps no caller pointer after a call returns, except the weight
 *     pointers given to ssd_create, which must stay valid until ssd_destroy.
 *   - cu_* arrays are HOST arrays of B+1 exclusive prefix sums with cu[0] = 0 (ragged batches are
 *     host-side knowledge of whoever batches the utterances).  They are read before the call returns.
 *   - Every call enqueues its work on the hipStream_t given to ssd_create and returns without
 *     waiting for the device.  Outputs are valid after the caller synchronises that stream.
 *   - Return value: SSD_OK or a negative ssd_status.  Argument errors are detected on the host
 *     before anything is launched, so on a non-zero return no output buffer has been written.
 *     ssd_last_error gives a message for the last failing call on that context.
 *   - Device memory is allocated only by ssd_create and ssd_set_ctc_head (re-laid-out weights, small
 *     tables) and freed by ssd_destroy.  All activations live in the caller-provided workspace
 *     (ssd_set_workspace).
 *   - One context must not be used from two host threads at once.
 */
#ifndef SSD_H
#define SSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ssd_ctx ssd_ctx;

enum ssd_status {
    SSD_OK = 0,
    SSD_EINVAL = -1,        /* NULL pointer, negative count, malformed cu_* array, id out of range   */
    SSD_ESHAPE = -2,        /* a size the kernels do not support (see each call)                     */
    SSD_EWORKSPACE = -3,    /* no workspace set, or it is smaller than ssd_workspace_bytes says      */
    SSD_EHIP = -4,          /* a HIP runtime call failed (message holds the HIP error string)        */
    SSD_EUNSUPPORTED = -5   /* dtype / feature not built                                             */
};

enum ssd_dtype { SSD_F32 = 0, SSD_BF16 = 1 };
/* Matrix-core operand type of an SSD_BF16 model (the paper's stack runs in bfloat16, Sec. 3.2).
 *   SSD_OP_F16  (default) activations are rounded to IEEE half (11 significant bits) where they enter a
 *               contraction; the bf16 weights are converted once to half times a per-tensor power of two
 *               (exact for every value within 31 binades of the tensor's largest; ssd_inexact_weights
 *               counts the rest).  Range 65504: stores saturate and raise SSD_FLAG_ACT_OVERFLOW.
 *   SSD_OP_BF16 activations are rounded to bfloat16 (8 significant bits, the range of fp32), the stored
 *               weights are the operands.  Same kernels and MFMA rate; about 8 times the rounding error. */
enum ssd_operand { SSD_OP_F16 = 0, SSD_OP_BF16 = 1 };

/* Decoder-only LLM: pre-norm RMSNorm, grouped-query causal attention with half-split rotary
 * embedding (component i paired with i + head_dim/2), SwiGLU MLP, no biases.
 * dtype is the storage type of every weight and of speech_emb.  SSD_F32 is all fp32.  SSD_BF16
 * runs the contractions on the 16-bit matrix cores with fp32 accumulation and an fp32 residual
 * stream; the matrix-core operand type is chosen with `operand` (enum ssd_operand): IEEE half by
 * default, bfloat16 on request.
 * Supported: head_dim 128 (bf16) or any multiple of 4 up to 128 (f32); n_q_heads a multiple of
 * n_kv_heads (at most 4 times for bf16); for bf16 d_model (<= 8192), (n_q_heads + 2 n_kv_heads)*head_dim
 * and vocab multiples of 256, d_ff a multiple of 128; for f32 d_model, d_ff, n_q_heads*head_dim multiples of 16 and d_model <= 1024. */
typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ff, vocab;
    float   rms_eps, rope_theta;
    int32_t dtype;            /* enum ssd_dtype */
    int32_t max_positions;    /* longest sequence (speech + prompt + draft rows of one utterance) */
    int32_t operand;          /* enum ssd_operand; ignored for SSD_F32 unless SSD_OP_BF16 (rejected) */
} ssd_model_cfg;

/* All matrices are row-major [out_features, in_features] (y = W x); per-layer members are HOST
 * arrays of n_layers DEVICE pointers.  lm_head may alias embed. */
typedef struct {
    const void *embed;                /* dev [vocab, d_model]                        */
    const void *const *wq;            /* dev [n_q_heads*head_dim, d_model] per layer */
    const void *const *wk;            /* dev [n_kv_heads*head_dim, d_model]          */
    const void *const *wv;            /* dev [n_kv_heads*head_dim, d_model]          */
    const void *const *wo;            /* dev [d_model, n_q_heads*head_dim]           */
    const void *const *w_gate;        /* dev [d_ff, d_model]                         */
    const void *const *w_up;          /* dev [d_ff, d_model]                         */
    const void *const *w_down;        /* dev [d_model, d_ff]                         */
    const void *const *norm_attn;     /* dev [d_model] RMSNorm gain before attention */
    const void *const *norm_mlp;      /* dev [d_model] RMSNorm gain before the MLP   */
    const void *norm_final;           /* dev [d_model]                               */
    const void *lm_head;              /* dev [vocab, d_model]                        */
} ssd_weights;

/* Create a context bound to `hip_stream` (a hipStream_t, NULL = default stream) on the current
 * device.  cfg and weights may both be NULL for a context that only runs ctc_gate.  With a model,
 * the projection weights are copied into library-owned layouts (fused QKV and gate/up; for
 * SSD_BF16 every matrix incl. lm_head as scaled half), which waits for the copies; embed, the
 * norm gains (and for SSD_F32 wo, w_down, lm_head) are read in place on every call. */
int ssd_create(ssd_ctx **out, const ssd_model_cfg *cfg, const ssd_weights *weights, void *hip_stream);
void ssd_destroy(ssd_ctx *ctx);
/* SSD_BF16 models: number of weight values (all projection matrices and lm_head) whose conversion to
 * half times the tensor's power of two was not exact.  A bf16 value keeps all of its 8 significant
 * bits when its magnitude is within 31 binades of the largest magnitude of its tensor; smaller ones are
 * rounded to the half subnormal grid (absolute error below 2^-39 of the tensor's largest magnitude).
 * 0 for SSD_F32 models and for every tensor drawn from a distribution of ordinary dynamic range. */
int64_t ssd_inexact_weights(const ssd_ctx *ctx);

/* Bytes of workspace needed for calls with at most max_frames CTC frames, max_tokens decoder rows
 * (sum over utterances of speech + prompt + draft), max_verify_rows draft tokens and max_utts
 * utterances (ctc_head_gate and qformer_pool are covered once their weights have been set: ask again after
 * ssd_set_ctc_head / ssd_set_qformer).  The workspace is a dev buffer, 256-byte aligned, handed over with
 * ssd_set_workspace and owned by the caller; it may be replaced between calls. */
size_t ssd_workspace_bytes(const ssd_ctx *ctx, int64_t max_frames, int64_t max_tokens,
                           int64_t max_verify_rows, int64_t max_utts);
int ssd_set_workspace(ssd_ctx *ctx, void *dev_ptr, size_t bytes);

const char *ssd_last_error(const ssd_ctx *ctx);

/* Conditions that only the device sees (they depend on data in device memory) do not fail a call: the
 * kernels repair them and raise a sticky flag.  ssd_device_flags waits for the stream, writes the flags
 * raised since the last call to *flags (host) and clears them.
 *   SSD_FLAG_TOKEN_CLAMPED  a prompt, draft or first_tok id outside [0, vocab) was clamped into range
 *   SSD_FLAG_ACT_OVERFLOW   SSD_BF16 models: an activation left the range of the matrix-core operand type
 *                           (|v| > 65504 for IEEE half, or NaN) at one of the points where the fp32 pipeline
 *                           rounds to it (RMSNorm output, rotated q / k and v, SiLU(gate)*up, K/V-cache rows) and
 *                           was stored saturated to +-65504, or a log-likelihood came out non-finite.  Results of
 *                           calls since the last read are then not the model's: re-run in fp32 or rescale. */
enum ssd_device_flag { SSD_FLAG_TOKEN_CLAMPED = 1, SSD_FLAG_ACT_OVERFLOW = 2 };
int ssd_device_flags(ssd_ctx *ctx, int32_t *flags /*host*/);

/* Measurement aid (no counterpart in the paper): times kernel launches with HIP events recorded on
 * the context's stream.  ssd_profile_select chooses what the following calls bracket: one class,
 * SSD_PROF_ALL, or SSD_PROF_OFF (default; no events are recorded).  It waits for the stream and
 * discards earlier samples.  ssd_profile_read waits for the stream, writes per class the summed
 * device time in milliseconds and the number of bracketed launches since the last select/read
 * (arrays of SSD_PROF_N_CLASSES entries, host memory), and clears the samples.  A span covers one
 * kernel launch, except SSD_PROF_GATE (the two gate kernels) and SSD_PROF_LMHEAD (LM head,
 * merge of partials and prefix scan). */
enum ssd_prof_class {
    SSD_PROF_OFF = -2, SSD_PROF_ALL = -1,
    SSD_PROF_GATE = 0, SSD_PROF_GEMM_QKV = 1, SSD_PROF_ATTN = 2, SSD_PROF_GEMM_O = 3,
    SSD_PROF_GEMM_GATE_UP = 4, SSD_PROF_GEMM_DOWN = 5, SSD_PROF_LMHEAD = 6, SSD_PROF_OTHER = 7,
    SSD_PROF_AR = 8,          /* one span per ar_fallback call */
    SSD_PROF_CTC_HEAD = 9,    /* one span per ctc_head_gate call */
    SSD_PROF_QFORMER = 10,    /* one span per qformer_pool call */
    SSD_PROF_N_CLASSES = 11
};
int ssd_profile_select(ssd_ctx *ctx, int kernel_class);
/* Measurement aid: runs `iters` rounds of 16 independent v_mfma_f32_16x16x32_f16 per wavefront on
 * pseudo-random register operands, eight wavefronts on every CU, no memory traffic, and reports the
 * sustained rate (TFLOP/s) and the shader clock observed meanwhile (GHz): the ceiling that power
 * and clock management leave for the matrix cores on this device.  Uses the first 513 KB of the
 * workspace and waits for the stream. */
int ssd_measure_mfma_ceiling(ssd_ctx *ctx, int iters, float *tflops /*host*/, float *shader_ghz /*host*/);
/* Measurement aid: reads `bytes` (rounded down to a multiple of 16) of the caller's device buffer
 * `iters` times with a plain streaming kernel (one workgroup of eight wavefronts per CU, each
 * walking its own contiguous share with eight 1 KB loads in flight per wavefront) and reports the sustained rate in GB/s: what this device delivers to a kernel that
 * does nothing but read, i.e. the practical ceiling under the nominal HBM peak for the gate and the
 * weight-streaming steps.  The buffer should be much larger than the 256 MB memory-side cache.
 * dev_buf: device pointer, 16-byte aligned, not written.  Needs a workspace (one word of it is
 * used) and waits for the stream.  Errors: SSD_EINVAL, SSD_EWORKSPACE, SSD_EHIP. */
int ssd_measure_hbm_read(ssd_ctx *ctx, const void *dev_buf, size_t bytes, int iters, float *gbytes_per_s /*host*/);
int ssd_profile_read(ssd_ctx *ctx, float *total_ms /*host [SSD_PROF_N_CLASSES]*/,
                     int32_t *launches /*host [SSD_PROF_N_CLASSES]*/);

/* Sec. 2.1.  For every frame t of every utterance: softmax over the V_ctc scores (blank included),
 * entropy H_t in nats (Eq. 3, left side) and greedy label a_t = lowest-index argmax of the stored
 * scores (Eq. 2).  Per utterance b (frames cu_frames[b] .. cu_frames[b+1]-1, at least one):
 *   draft  = B(a): merge consecutive duplicates, then drop blank_id; written to
 *            draft_ctc[cu_frames[b] ...], its length to draft_len[b];
 *   max_entropy[b] = max_t H_t;  gate_pass[b] = 1 iff max_entropy[b] < tau_ctc (strict, Eq. 3).
 * logits: dev [cu_frames[B], V_ctc] packed rows, row-major, dtype SSD_F32 or SSD_BF16; -inf is a
 * legal score (probability 0), NaN/+inf give unspecified results.
 * frame_entropy / frame_argmax: optional dev outputs [cu_frames[B]] (NULL to skip). */
int ctc_gate(ssd_ctx *ctx, const void *logits, int dtype, const int32_t *cu_frames /*host*/, int B,
             int V_ctc, int blank_id, float tau_ctc,
             float *frame_entropy, int32_t *frame_argmax,
             float *max_entropy /*dev [B]*/, uint8_t *gate_pass /*dev [B]*/,
             int32_t *draft_ctc /*dev [cu_frames[B]]*/, int32_t *draft_len /*dev [B]*/);

/* ctc_gate for callers that cannot allocate: code under HIP graph capture, tight serving loops and
 * harnesses that forbid allocation.  Needs no context and no workspace; calls no hipMalloc, hipFree,
 * host allocation, copy or wait: it only launches the two kernels of ctc_gate on `hip_stream`
 * (a hipStream_t, NULL = default stream) of the current device.  The per-frame entropies and greedy
 * labels, which ctc_gate keeps in the workspace, live in a device array built into the library:
 * 8 bytes per frame, SSD_NOALLOC_MAX_FRAMES frames (2 MiB), one copy per GPU for the life of the process.
 * Differences from ctc_gate: cu_frames_dev is a DEVICE array of B+1 prefix sums (the host cannot check
 * it: the kernels clamp every utterance's frame range into [0, n_frames], so a malformed array gives
 * wrong results for that utterance but no access outside the buffers); n_frames (= cu_frames_dev[B]) is
 * passed explicitly; frame_entropy / frame_argmax are not returned.  Outputs as for ctc_gate and, for
 * well-formed prefix sums, bit-identical to it.
 * Errors (nothing is launched): SSD_EINVAL (NULL pointer, B, n_frames or V_ctc <= 0, blank_id out of
 * range), SSD_EUNSUPPORTED (dtype), SSD_ESHAPE (n_frames > SSD_NOALLOC_MAX_FRAMES), SSD_EHIP.  `err`
 * (host, may be NULL) receives a message of at most err_len bytes.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 * streams or host threads) race; calls on one stream are ordered and safe. */
#define SSD_NOALLOC_MAX_FRAMES 262144
int ctc_gate_noalloc(void *hip_stream, const void *logits /*dev [n_frames, V_ctc]*/, int dtype,
                     const int32_t *cu_frames_dev /*dev [B+1]*/, int B, int64_t n_frames, int V_ctc, int blank_id,
                     float tau_ctc, float *max_entropy /*dev [B]*/, uint8_t *gate_pass /*dev [B]*/,
                     int32_t *draft_ctc /*dev [n_frames]*/, int32_t *draft_len /*dev [B]*/,
                     char *err /*host*/, size_t err_len);

/* Sec. 3.1 (output layer of the CTC encoder: 1024-wide states, 348 symbols) feeding Sec. 2.1.
 * ssd_set_ctc_head copies the output layer into the context (padded to a multiple of 128
 * symbols; the caller's arrays may be released on return; a second call replaces the first).
 * w_ctc: dev [V_ctc, d_enc] bfloat16 row-major; bias: dev [V_ctc] fp32 or NULL (zero);
 * d_enc a multiple of 64, V_ctc <= 65536.  Allocates device memory; waits for the stream.
 *
 * ctc_head_gate evaluates z[t, v] = enc_h[t] . w_ctc[v] + bias[v] and, on those scores, exactly what
 * ctc_gate defines (Eqs. 2-3 and the collapse B) with the same outputs.  The scores are formed in
 * fp32 from the stored bf16 operands and are never rounded or written to memory; the argmax is taken
 * on the fp32 scores (lowest index among equal ones).
 * enc_h: dev [cu_frames[B], d_enc] bfloat16 packed rows.  Other arguments as for ctc_gate.
 * Errors: SSD_EINVAL (no output layer set, NULL or inconsistent arguments), SSD_EWORKSPACE. */
int ssd_set_ctc_head(ssd_ctx *ctx, const void *w_ctc, const float *bias, int V_ctc, int d_enc);
int ctc_head_gate(ssd_ctx *ctx, const void *enc_h, const int32_t *cu_frames /*host*/, int B, int blank_id,
                  float tau_ctc, float *frame_entropy, int32_t *frame_argmax, float *max_entropy,
                  uint8_t *gate_pass, int32_t *draft_ctc, int32_t *draft_len);

/* Sec. 3.1 (projector): the windowed cross-attention that turns encoder frames into the acoustic embeddings g of
 * Sec. 2.2: every window of `window` (15) consecutive frames of an utterance is summarised by n_q (3) trainable
 * queries, a downsampling by 5.  ssd_set_qformer copies the weights into the context (allocates device memory;
 * waits for the stream; the caller's arrays may be released on return; a second call replaces the first):
 *   q_proj dev [n_q, d_h] bf16       the queries after their query projection (constants of the model)
 *   w_k, w_v dev [d_h, d_enc] bf16   key and value projections of the frames
 *   w_o dev [d_out, d_h] bf16        output projection (d_out = d_model of the LLM)
 * n_heads heads of d_h / n_heads dims, scores scaled by 1 / sqrt(d_head).  Limits: n_q <= 4, n_q * n_heads <= 64,
 * window <= 32, d_h a multiple of 64 and of 4 * n_heads, d_enc of 64, d_out of 256 (SSD_ESHAPE otherwise).
 * The key projection is folded into n_q * n_heads score rows at this point (the queries are constants).
 *
 * qformer_pool: for every utterance b and window w of its frames (the last one may be shorter and attends over
 * the frames it has), query j: p = softmax over the window's frames of the head-wise scores, o = sum_t p_t w_v h_t,
 * g = w_o o, written as bf16 to speech_emb row cu_speech[b] + n_q * w + j (the projected values w_v h_t pass through
 * IEEE half on the way: one beyond 65504 is clamped and raises SSD_FLAG_ACT_OVERFLOW); cu_speech (host, B + 1 entries) is
 * filled with the prefix sums S_b = n_q * ceil(T_b / window) that verify_forward takes.  The rest of a q-former
 * layer (self-attention among the queries, feed-forward block, normalisation, second layer) is not described in
 * the paper and not part of this call.
 * enc_h: dev [cu_frames[B], d_enc] bf16 packed rows; speech_emb: dev [n_q * (frames / window + B), d_out] is enough.
 * Needs the workspace ssd_workspace_bytes reports after ssd_set_qformer.  Errors: SSD_EINVAL, SSD_ESHAPE, SSD_EWORKSPACE. */
int ssd_set_qformer(ssd_ctx *ctx, const void *q_proj, const void *w_k, const void *w_v, const void *w_o, int n_q,
                    int n_heads, int d_h, int d_enc, int d_out, int window);
int qformer_pool(ssd_ctx *ctx, const void *enc_h, const int32_t *cu_frames /*host*/, int B, void *speech_emb,
                 int32_t *cu_speech /*host, out*/);

/* Between Sec. 2.1 and Sec. 2.2 (Eq. 7: only utterances that fail the entropy gate are verified).  Packs the
 * verification inputs of the n_sel selected utterances (sel: host, indices into the batch of B utterances, in
 * the order they will be verified) on the device:
 *   speech_out  [sum S, d_model]  rows of speech_all (dev [cu_speech_all[B], d_model], dtype SSD_F32 / SSD_BF16)
 *   prompt_out  [sum P]           entries of prompt_all (dev)
 *   draft_ids_out [sum U]         ctc_to_llm[draft_ctc[cu_frames[b] + i]], i < draft_len[b]: the draft of ctc_gate
 *                                 re-expressed in LLM token ids through a caller-supplied table (dev [V_ctc]; the
 *                                 paper leaves re-tokenisation to its software stack; NULL copies the ids unchanged)
 * and writes the matching prefix sums cu_speech_out / cu_prompt_out / cu_draft_out (host [n_sel + 1]) that
 * verify_forward and accept_prefix take.  cu_frames, draft_len (host copy of ctc_gate's output), cu_speech_all and
 * cu_prompt_all are host arrays over all B utterances.  Output buffers are the caller's (sizes as above; the sums
 * are known on the host before the call).  Uses 4 bytes of workspace per output row / id.
 * Errors: SSD_EINVAL, SSD_ESHAPE (a speech row is not a multiple of 16 bytes), SSD_EWORKSPACE. */
int ssd_select_unconfident(ssd_ctx *ctx, int B, int n_sel, const int32_t *sel /*host*/, const int32_t *cu_frames /*host*/,
                           const int32_t *draft_len /*host [B]*/, const int32_t *draft_ctc /*dev*/,
                           const int32_t *ctc_to_llm /*dev [V_ctc] or NULL*/, int V_ctc,
                           const void *speech_all /*dev*/, const int32_t *cu_speech_all /*host*/,
                           const int32_t *prompt_all /*dev*/, const int32_t *cu_prompt_all /*host*/, int d_model, int dtype,
                           void *speech_out /*dev*/, int32_t *prompt_out /*dev*/, int32_t *draft_ids_out /*dev*/,
                           int32_t *cu_speech_out /*host*/, int32_t *cu_prompt_out /*host*/, int32_t *cu_draft_out /*host*/);

/* out[i] = src[idx[i]] for i < n on the device (src, out: dev int32; idx: host, non-negative, in range of src:
 * the host cannot check the upper end).  The glue for picking token ids out of device arrays without a round
 * trip, e.g. first_tok of ar_fallback = greedy_tok at each utterance's first rejected position.  Uses 4 n bytes
 * of workspace. */
int ssd_gather_i32(ssd_ctx *ctx, const int32_t *src /*dev*/, const int32_t *idx /*host [n]*/, int n, int32_t *out /*dev [n]*/);

/* Sec. 2.2 (Eq. 4; parallel scoring through the causal mask).  For each of the Bv utterances that
 * did not pass the gate, runs the decoder over the rows [speech_emb rows; embed[prompt ids];
 * embed[draft ids]] at positions 0..n-1 and writes, for draft token i = 1..U, the final-RMSNormed
 * hidden row of sequence index S + P + i - 2 (the position whose next-token distribution scores
 * token i) to h_verify row cu_draft[b] + i - 1.  An utterance needs S + P >= 1; U = 0 is legal.
 * speech_emb: dev [cu_speech[Bv], d_model]; prompt_ids / draft_ids: dev int32 LLM token ids
 * (ids outside [0, vocab) are clamped on the device); h_verify: dev [cu_draft[Bv], d_model], in the operand
 * type for SSD_BF16 models (IEEE half or bfloat16) and fp32 for SSD_F32: an activation buffer that
 * accept_prefix consumes.
 * SSD_ESHAPE if an activation matrix of the call (rows x max(d_ff, q+k+v width, d_model) elements) would
 * reach 4 GiB: split the batch. */
int verify_forward(ssd_ctx *ctx, const void *speech_emb, const int32_t *cu_speech /*host*/,
                   const int32_t *prompt_ids, const int32_t *cu_prompt /*host*/,
                   const int32_t *draft_ids, const int32_t *cu_draft /*host*/, int Bv,
                   void *h_verify);

/* The same pass, additionally storing the rotated keys and the values of every row of every layer
 * into the K/V cache set with ssd_set_kv_cache, so that ar_fallback can continue from any prefix of
 * the sequence: row `pos` of utterance b goes to cache slot kv_start[b] + pos.  kv_start: host [Bv];
 * the slot ranges of different utterances must not overlap and should leave room for the tokens
 * ar_fallback will append. */
int verify_forward_kv(ssd_ctx *ctx, const void *speech_emb, const int32_t *cu_speech /*host*/,
                      const int32_t *prompt_ids, const int32_t *cu_prompt /*host*/,
                      const int32_t *draft_ids, const int32_t *cu_draft /*host*/, int Bv,
                      const int32_t *kv_start /*host*/, void *h_verify);

/* K/V cache for the auto-regressive fallback: a caller-owned dev buffer, 256-byte aligned, holding
 * for every layer K [slots, n_kv_heads*head_dim] and V [slots, ...] in the activation type (the operand
 * type for SSD_BF16 models, fp32 for SSD_F32).  A NULL pointer detaches the cache. */
size_t ssd_kv_cache_bytes(const ssd_ctx *ctx, int64_t slots);
int ssd_set_kv_cache(ssd_ctx *ctx, void *dev_ptr, size_t bytes, int64_t slots);

/* Sec. 2.3, Eq. 6: greedy auto-regressive continuation of Br utterances from their accepted
 * prefixes.  Utterance b has ctx_len[b] = S + P + accept_len valid rows in the cache starting at slot
 * kv_start[b] (written by verify_forward_kv; rows beyond the prefix are overwritten here).
 * first_tok[b] (dev) is the token at position ctx_len[b]: the model's own choice after the prefix,
 * which accept_prefix already delivers as greedy_tok at the first rejected draft position.
 * Step t = 0..n_steps-1 feeds token u_t (u_0 = first_tok) at position ctx_len + t, appends its keys and
 * values to the cache and writes u_{t+1} = lowest-index argmax of the next-token distribution to
 * out_tokens[t * Br + b] (dev, [n_steps, Br]).  Stopping at an end-of-sequence token is the caller's
 * business (truncate the row).  Needs ssd_ar_workspace_bytes(ctx, Br, n_steps) bytes of workspace.
 * head_dim must be a multiple of 8 (SSD_ESHAPE otherwise). */
size_t ssd_ar_workspace_bytes(const ssd_ctx *ctx, int max_utts, int max_steps);
int ar_fallback(ssd_ctx *ctx, int Br, const int32_t *kv_start /*host [Br]*/, const int32_t *ctx_len /*host [Br]*/,
                const int32_t *first_tok /*dev [Br]*/, int n_steps, int32_t *out_tokens /*dev [n_steps, Br]*/);

/* Sec. 3.2-3.3: operating points.  Frame entropies and token likelihoods do not depend on the
 * thresholds, so the decisions for a whole grid of (tau_CTC, tau_SLM) come from one gate pass and one
 * verification pass.  tau arrays are host arrays; outputs are dev, threshold-major:
 * gate_pass[a*B + b] = max_entropy[b] < tau_ctc[a];  accept_len / all_accepted[a*Bv + b] as in
 * accept_prefix with tau_slm[a].  The ablations of Sec. 3.3 are caller policy on these outputs:
 * gate only = skip the verification calls; verification only = verify every utterance and ignore
 * gate_pass.  Both calls use a few hundred bytes at the start of the workspace. */
int ssd_gate_grid(ssd_ctx *ctx, const float *max_entropy /*dev [B]*/, int B, const float *tau_ctc /*host*/, int n_tau,
                  uint8_t *gate_pass /*dev [n_tau, B]*/);
int ssd_accept_grid(ssd_ctx *ctx, const float *draft_logp /*dev*/, const int32_t *cu_draft /*host*/, int Bv,
                    const float *tau_slm /*host*/, int n_tau, int32_t *accept_len /*dev [n_tau, Bv]*/,
                    uint8_t *all_accepted /*dev [n_tau, Bv]*/);

/* Sec. 3.2: length-sorted adaptive batching under a token budget (the paper uses 50K).  Host only,
 * no context.  lengths[i] > 0 is the row count of utterance i (CTC frames for the gate phase,
 * speech + prompt + draft rows for verification, context rows for the fallback phase: the phases
 * are batched separately).  Utterances are taken longest first (ties: lower index first) and added to
 * the current batch while its cost stays <= max_tokens; cost = sum of lengths (packed rows, what this
 * library runs) or, with padded != 0, size x longest member (what a padded implementation pays).
 * An utterance longer than the budget forms a batch of its own.  Outputs: order[n] (utterance
 * indices in batch order), batch_start[n_batches + 1] (needs room for n + 1 entries), n_batches. */
int ssd_plan_batches(const int32_t *lengths, int n, int64_t max_tokens, int padded, int32_t *order,
                     int32_t *batch_start, int32_t *n_batches);

/* Sec. 2.2-2.3 (Eq. 5, definition of j, Eq. 7).  draft_logp[r] = log softmax(lm_head . h_verify[r])
 * at token draft_ids[r]; the logits are never written to memory.  Token i passes iff
 * draft_logp > ln(tau_slm), evaluated in fp32 with ln(tau_slm) rounded from double (tau_slm <= 0
 * accepts everything).  accept_len[b] = j - 1 where j is the first failing token, or U if none;
 * all_accepted[b] = (accept_len[b] == U).  greedy_tok (optional, NULL to skip) receives the
 * lowest-index argmax over the vocabulary at every row: the token greedy decoding would emit there. */
int accept_prefix(ssd_ctx *ctx, const void *h_verify, const int32_t *draft_ids /*dev*/,
                  const int32_t *cu_draft /*host*/, int Bv, float tau_slm,
                  float *draft_logp /*dev [cu_draft[Bv]]*/, int32_t *accept_len /*dev [Bv]*/,
                  uint8_t *all_accepted /*dev [Bv]*/, int32_t *greedy_tok /*dev [cu_draft[Bv]] or NULL*/);

#ifdef __cplusplus
}
#endif
#endif /* SSD_H */
