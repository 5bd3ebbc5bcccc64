"""CPU oracle for the gate -> verify -> accept path of CTC-draft self-speculative decoding.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module:
it exists so that tests, the smoke check and the benchmark's CPU-baseline leg have
a plain, slow, obviously-correct evaluation of the paper's definitions to compare
the HIP kernels with.  It shares no code with the HIP path and never calls it.

Precision: every input (CTC logits, weights, embeddings) is taken at its stored
value, converted exactly to float64, and all arithmetic is float64 numpy.  The
method on this path is exact (no approximation), so each function is the paper's
definition written out; utterances are processed one at a time.

Pins: every function below is checked in tests/test_oracle_*.py against closed
forms, library routines, invariants and brute force.  One caveat, also stated
there: the absolute values of draft log-likelihoods on the large random-init
configurations have no pin beyond those checks on reduced shapes (parity unpinned
in absolute value for full-size models; the arithmetic is the same code path).

Readings of points the paper leaves open are listed beside each function.
"""
import math
from typing import Dict, List, Sequence

import numpy as np


# --------------------------------------------------------------------------- gate

def _check_logits(z: np.ndarray) -> None:
    if np.isnan(z).any() or np.isposinf(z).any():
        raise ValueError("CTC logits contain NaN or +inf: the gate is undefined")


def frame_entropy(z: np.ndarray) -> np.ndarray:
    """Entropy of the CTC output distribution of every frame (left side of Eq. 3, Sec. 2.1).

    z: [T, V] unnormalised log-scores over the augmented vocabulary (blank included).
    p = softmax(z); H_t = sum_a -p(a) log p(a), natural log, with 0 log 0 = 0.
    """
    z = np.asarray(z, dtype=np.float64)
    _check_logits(z)
    m = z.max(axis=1, keepdims=True)
    e = np.exp(z - m)
    s = e.sum(axis=1, keepdims=True)
    p = e / s
    logp = (z - m) - np.log(s)
    with np.errstate(invalid="ignore"):
        terms = np.where(p > 0.0, -p * logp, 0.0)
    return terms.sum(axis=1)


def greedy_alignment(z: np.ndarray) -> np.ndarray:
    """Greedy alignment path (Eq. 2, Sec. 2.1): per-frame argmax over the augmented vocabulary.

    Softmax is monotone, so the argmax is taken on the stored scores.  Ties: lowest index.
    """
    z = np.asarray(z, dtype=np.float64)
    _check_logits(z)
    return np.argmax(z, axis=1).astype(np.int32)     # numpy returns the first maximum


def collapse(path: Sequence[int], blank: int) -> np.ndarray:
    """The map B of Sec. 2.1: remove consecutive duplicates, then remove blanks, in this order."""
    no_dup: List[int] = []
    for a in path:
        if not no_dup or a != no_dup[-1]:
            no_dup.append(int(a))
    return np.asarray([a for a in no_dup if a != blank], dtype=np.int32)


def collapse_streaming(path: Sequence[int], blank: int) -> np.ndarray:
    """Same map as `collapse`, one frame at a time: keep a frame iff it is not blank and it
    differs from the frame before it.  Kept only to cross-check `collapse`."""
    out, prev = [], None
    for a in path:
        if a != blank and a != prev:
            out.append(int(a))
        prev = a
    return np.asarray(out, dtype=np.int32)


def ctc_gate(logits: np.ndarray, cu_frames: Sequence[int], blank: int, tau_ctc: float) -> Dict:
    """Gate of Sec. 2.1: draft = B(greedy path); accepted as final iff every frame entropy
    is strictly below tau_ctc (Eq. 3).  Utterance b owns rows cu_frames[b]:cu_frames[b+1]."""
    logits = np.asarray(logits, dtype=np.float64)
    H = frame_entropy(logits) if len(logits) else np.zeros(0)
    a = greedy_alignment(logits) if len(logits) else np.zeros(0, np.int32)
    B = len(cu_frames) - 1
    drafts, max_h, gate = [], np.zeros(B), np.zeros(B, dtype=bool)
    for b in range(B):
        lo, hi = int(cu_frames[b]), int(cu_frames[b + 1])
        if hi <= lo:
            raise ValueError("utterance without frames")
        drafts.append(collapse(a[lo:hi], blank))
        max_h[b] = H[lo:hi].max()
        gate[b] = bool(np.all(H[lo:hi] < tau_ctc))
    return {"frame_entropy": H, "frame_argmax": a, "max_entropy": max_h,
            "gate_pass": gate, "drafts": drafts}


# --------------------------------------------------------------------------- CTC output layer

def ctc_head_logits(enc_h, w_ctc, bias=None) -> np.ndarray:
    """Scores of the CTC output layer (Sec. 3.1: the encoder's 1024-wide states feed an output
    layer over the 348 CTC symbols): z_t = W h_t + b.

    enc_h: [T, d_enc], w_ctc: [V, d_enc], bias: [V] or None.  Stored values widened exactly to
    float64; one library matrix product.
    """
    z = _f64(enc_h) @ _f64(w_ctc).T
    if bias is not None:
        z = z + _f64(bias)[None, :]
    return z


def ctc_head_gate(enc_h, w_ctc, bias, cu_frames: Sequence[int], blank: int, tau_ctc: float) -> Dict:
    """Eqs. 2-3 evaluated on the scores of the output layer (never rounded to a storage type)."""
    return ctc_gate(ctc_head_logits(enc_h, w_ctc, bias), cu_frames, blank, tau_ctc)


# ------------------------------------------------------------------ projector windows

def qformer_window_pool(enc_h, cu_frames: Sequence[int], q_proj, w_k, w_v, w_o, n_heads: int, window: int = 15):
    """Windowed cross-attention of the query-transformer projector (Sec. 3.1: every window of 15 consecutive
    frames is summarised by 3 trainable queries, a downsampling of the acoustic embeddings by 5).

    enc_h  [sum_T, d_enc]  encoder states, utterance b owns rows cu_frames[b] .. cu_frames[b+1]-1
    q_proj [n_q, d_h]      the trainable queries after their query projection (constants of the model)
    w_k, w_v [d_h, d_enc]  key / value projections of the frames;  w_o [d_out, d_h]  output projection
    For every utterance and every window w (frames 15 w .. 15 w + 14 of the utterance; the last window may be
    shorter and attends over the frames it has), query j and head h (d_head = d_h / n_heads):
        s_t = q_proj[j, head h] . (w_k enc_h[t])[head h] / sqrt(d_head),   p = softmax_t(s),
        o[j, head h] = sum_t p_t (w_v enc_h[t])[head h],                   g[j] = w_o o[j].
    Returns (g [sum_S, d_out], cu_speech) with S_b = n_q * ceil(T_b / window): the rows an utterance hands to
    the LLM as speech embeddings, in window order, queries of a window next to each other.
    Readings: the paper names the window, the query count and the rate only; the rest of a q-former layer
    (self-attention among the queries, feed-forward block, normalisation, the second layer) is not described
    and not part of this function; windows never cross an utterance boundary.
    """
    H = _f64(enc_h)
    Q, Wk, Wv, Wo = _f64(q_proj), _f64(w_k), _f64(w_v), _f64(w_o)
    n_q, d_h = Q.shape
    if d_h % n_heads:
        raise ValueError("d_h must be a multiple of n_heads")
    dh = d_h // n_heads
    rows, cu_speech = [], [0]
    for b in range(len(cu_frames) - 1):
        lo, hi = int(cu_frames[b]), int(cu_frames[b + 1])
        if hi <= lo:
            raise ValueError("an utterance needs at least one frame")
        for w0 in range(lo, hi, window):
            Hw = H[w0:min(w0 + window, hi)]
            K, V = Hw @ Wk.T, Hw @ Wv.T
            o = np.zeros((n_q, d_h))
            for h in range(n_heads):
                sl = slice(h * dh, (h + 1) * dh)
                s = (Q[:, sl] @ K[:, sl].T) / math.sqrt(dh)          # [n_q, frames of the window]
                s = s - s.max(axis=1, keepdims=True)
                p = np.exp(s)
                p = p / p.sum(axis=1, keepdims=True)
                o[:, sl] = p @ V[:, sl]
            rows.append(o @ Wo.T)
        cu_speech.append(cu_speech[-1] + n_q * (-(-(hi - lo) // window)))
    return np.concatenate(rows, axis=0), np.asarray(cu_speech, dtype=np.int32)


# ------------------------------------------------------------------------ decoder

def rmsnorm(x: np.ndarray, w: np.ndarray, eps: float) -> np.ndarray:
    """x * w / sqrt(mean(x^2) + eps) over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * w


def rope(v: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary position embedding, half-split pairing: component i is paired with i + hd/2
    and the pair is rotated by angle pos * theta^(-2i/hd).  v: [n, heads, hd]."""
    hd = v.shape[-1]
    half = hd // 2
    inv = theta ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = pos.astype(np.float64)[:, None] * inv[None, :]          # [n, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = v[..., :half], v[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(t: np.ndarray) -> np.ndarray:
    return t / (1.0 + np.exp(-t))


def decoder_layer(x: np.ndarray, L: Dict[str, np.ndarray], cfg) -> np.ndarray:
    """One pre-norm decoder layer on a single utterance x: [n, d] (positions 0..n-1).

    Causal self-attention with grouped KV heads (query head h reads KV head
    h // (n_q_heads / n_kv_heads)), then SwiGLU MLP, both with residual connections.
    This is the network whose next-token distribution Eq. 4 (Sec. 2.2) factorises.
    """
    n = x.shape[0]
    hq, hkv, hd = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    pos = np.arange(n)
    a = rmsnorm(x, L["norm_attn"], cfg.rms_eps)
    q = rope((a @ L["wq"].T).reshape(n, hq, hd), pos, cfg.rope_theta)
    k = rope((a @ L["wk"].T).reshape(n, hkv, hd), pos, cfg.rope_theta)
    v = (a @ L["wv"].T).reshape(n, hkv, hd)
    o = np.zeros((n, hq, hd))
    group = hq // hkv
    future = np.triu(np.ones((n, n), dtype=bool), k=1)
    for h in range(hq):
        g = h // group
        s = (q[:, h, :] @ k[:, g, :].T) / math.sqrt(hd)
        s = np.where(future, -np.inf, s)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=1, keepdims=True)
        o[:, h, :] = p @ v[:, g, :]
    x = x + o.reshape(n, hq * hd) @ L["wo"].T
    b = rmsnorm(x, L["norm_mlp"], cfg.rms_eps)
    x = x + (silu(b @ L["w_gate"].T) * (b @ L["w_up"].T)) @ L["w_down"].T
    return x


def _f64(t) -> np.ndarray:
    """Exact widening of a stored tensor (numpy array or torch tensor, any float type)."""
    if isinstance(t, np.ndarray):
        return t.astype(np.float64)
    return t.detach().double().cpu().numpy()      # widen where the tensor lives, then copy


def decoder_hidden(xs: List[np.ndarray], weights: Dict, cfg) -> List[np.ndarray]:
    """Residual stream after the last layer for each utterance in xs (list of [n_b, d]).
    Layers are the outer loop only so that a layer's weights are widened once."""
    xs = [np.array(x, dtype=np.float64) for x in xs]
    for L in weights["layers"]:
        L64 = {k: _f64(v) for k, v in L.items()}
        xs = [decoder_layer(x, L64, cfg) for x in xs]
    return xs


def assemble_inputs(weights: Dict, speech_emb, cu_speech, prompt_ids, cu_prompt,
                    draft_ids, cu_draft) -> List[np.ndarray]:
    """Input rows of each utterance: [speech embeddings g; E[prompt]; E[draft]] (Sec. 2.2:
    the LLM is conditioned on g and on the draft prefix)."""
    E = weights["embed"]
    sp = _f64(speech_emb)
    xs = []
    for b in range(len(cu_draft) - 1):
        pid = np.asarray(prompt_ids[cu_prompt[b]:cu_prompt[b + 1]], dtype=np.int64)
        did = np.asarray(draft_ids[cu_draft[b]:cu_draft[b + 1]], dtype=np.int64)
        rows = [sp[cu_speech[b]:cu_speech[b + 1]]]
        if len(pid):
            rows.append(_f64(E[pid]))
        if len(did):
            rows.append(_f64(E[did]))
        xs.append(np.concatenate(rows, axis=0))
    return xs


def lm_head_logp(h: np.ndarray, w_lm: np.ndarray, target: int):
    """Eq. 5 at one scoring position: log-softmax over the whole vocabulary of the logits w_lm @ h, read at
    the target id; also the greedy token (lowest-index argmax).  h: final-normed hidden row."""
    logits = w_lm @ h
    mx = logits.max()
    lse = mx + math.log(np.exp(logits - mx).sum())
    return float(logits[target] - lse), int(np.argmax(logits))


def draft_logp(weights: Dict, cfg, speech_emb, cu_speech, prompt_ids, cu_prompt,
               draft_ids, cu_draft, return_hidden: bool = False, return_greedy: bool = False):
    """log p(y_i | y_<i, g) for every draft token (the quantity thresholded in Eq. 5, Sec. 2.2).

    Draft token i (1-based) of an utterance with S speech rows and P prompt rows is scored
    by the output distribution at sequence index S + P + i - 2, i.e. the position just
    before the token.  All positions come from one causal forward over the whole sequence.
    Returns a list with one float64 array of length U_b per utterance; optionally also the
    final-normed hidden rows and the greedy token (lowest-index argmax over the vocabulary)
    of each scoring position.
    """
    xs = assemble_inputs(weights, speech_emb, cu_speech, prompt_ids, cu_prompt, draft_ids, cu_draft)
    hs = decoder_hidden(xs, weights, cfg)
    w_f, w_lm = _f64(weights["norm_final"]), _f64(weights["lm_head"])
    out, hid, greedy = [], [], []
    for b, x in enumerate(hs):
        S = int(cu_speech[b + 1] - cu_speech[b])
        P = int(cu_prompt[b + 1] - cu_prompt[b])
        y = np.asarray(draft_ids[cu_draft[b]:cu_draft[b + 1]], dtype=np.int64)
        lp = np.zeros(len(y))
        hv = np.zeros((len(y), x.shape[1]))
        gt = np.zeros(len(y), dtype=np.int32)
        for i in range(1, len(y) + 1):
            if S + P + i - 2 < 0:
                raise ValueError("first draft token has no conditioning position")
            h = rmsnorm(x[S + P + i - 2], w_f, cfg.rms_eps)
            lp[i - 1], gt[i - 1] = lm_head_logp(h, w_lm, int(y[i - 1]))
            hv[i - 1] = h
        out.append(lp)
        hid.append(hv)
        greedy.append(gt)
    if not (return_hidden or return_greedy):
        return out
    res = [out]
    if return_hidden:
        res.append(hid)
    if return_greedy:
        res.append(greedy)
    return tuple(res)


def ar_fallback(weights: Dict, cfg, speech_emb_b, prompt_ids_b, prefix_ids_b, n_steps: int) -> np.ndarray:
    """Greedy auto-regressive continuation from an accepted prefix (Sec. 2.3, Eq. 6, for one utterance).

    The sequence [speech; prompt; prefix] is extended one token at a time; every token is the
    lowest-index argmax of the next-token distribution at the last position.  Plain and quadratic:
    the whole forward is recomputed for every token (no cache).  Returns n_steps + 1 tokens: the
    first is the model's own choice right after the prefix (the token that replaces the first
    rejected draft token), the rest continue from it.
    """
    w_f, w_lm = _f64(weights["norm_final"]), _f64(weights["lm_head"])
    sp = _f64(speech_emb_b)
    ids = [int(t) for t in list(prompt_ids_b) + list(prefix_ids_b)]
    if len(sp) + len(ids) < 1:
        raise ValueError("nothing to condition on")
    out = []
    for _ in range(n_steps + 1):
        idx = np.asarray(ids, dtype=np.int64)
        rows = [sp] + ([_f64(weights["embed"][idx])] if len(idx) else [])
        x = decoder_hidden([np.concatenate(rows, axis=0)], weights, cfg)[0]
        h = rmsnorm(x[-1], w_f, cfg.rms_eps)
        tok = int(np.argmax(w_lm @ h))
        out.append(tok)
        ids.append(tok)
    return np.asarray(out, dtype=np.int32)


# ------------------------------------------------------------------------ accept

def accept_prefix(logp: Sequence[float], tau_slm: float) -> Dict:
    """Relaxed acceptance (Eq. 5, Sec. 2.2) and longest verified prefix (Sec. 2.3).

    Token i passes iff p_i > tau_slm (strict).  j = min{i : p_i <= tau_slm}; the accepted
    prefix is y_<j, of length j - 1; if no token fails the whole draft (length U) is accepted.
    The comparison is done on log-likelihoods: log p_i > ln tau.  tau <= 0 accepts everything,
    an empty draft is accepted vacuously.
    """
    ln_tau = math.log(tau_slm) if tau_slm > 0 else -math.inf
    U = len(logp)
    j = None
    for i in range(1, U + 1):
        if not (logp[i - 1] > ln_tau):
            j = i
            break
    n_acc = U if j is None else j - 1
    return {"accept_len": n_acc, "all_accepted": n_acc == U}


def threshold_grid(max_entropy: Sequence[float], logps: List[Sequence[float]], taus_ctc: Sequence[float],
                   taus_slm: Sequence[float]) -> Dict:
    """Decisions for a grid of operating points (Sec. 3.2: tau_CTC in [0.7, 3.0], tau_SLM in {0.1, 0.2}).
    Frame entropies and token likelihoods do not depend on the thresholds, so every grid point is the
    single-threshold rule applied to the same numbers."""
    gate = np.array([[bool(h < t) for h in max_entropy] for t in taus_ctc], dtype=bool).reshape(len(taus_ctc), len(max_entropy))
    acc = np.array([[accept_prefix(lp, t)["accept_len"] for lp in logps] for t in taus_slm], dtype=np.int32).reshape(len(taus_slm), len(logps))
    full = np.array([[accept_prefix(lp, t)["all_accepted"] for lp in logps] for t in taus_slm], dtype=bool).reshape(len(taus_slm), len(logps))
    return {"gate_pass": gate, "accept_len": acc, "all_accepted": full}


def plan_batches(lengths: Sequence[int], max_tokens: int, padded: bool) -> List[List[int]]:
    """Length-sorted adaptive batching under a token budget (Sec. 3.2).

    Utterances are taken longest first (ties: lower index first) and appended to the current batch
    while the batch stays within max_tokens; the cost of a batch is the sum of its lengths (packed
    rows) or, with padded=True, its size times its longest member.  A single utterance longer than
    the budget forms a batch of its own.  Returns lists of utterance indices.
    """
    order = sorted(range(len(lengths)), key=lambda i: (-int(lengths[i]), i))
    batches: List[List[int]] = []
    cur: List[int] = []
    for i in order:
        cand = cur + [i]
        cost = (len(cand) * max(int(lengths[k]) for k in cand)) if padded else sum(int(lengths[k]) for k in cand)
        if cur and cost > max_tokens:
            batches.append(cur)
            cur = [i]
        else:
            cur = cand
    if cur:
        batches.append(cur)
    return batches


def final_hypothesis_case(gate_pass: bool, all_accepted: bool) -> str:
    """Case split of Eq. 7 (Sec. 2.3): the draft is final if Eq. 3 or Eq. 5 holds, otherwise
    the accepted prefix is continued auto-regressively."""
    return "draft" if (gate_pass or all_accepted) else "prefix+ar"
