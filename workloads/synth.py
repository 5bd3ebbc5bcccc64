"""Seeded generators for the synthetic workloads.

Nothing here computes anything the method defines; the functions only draw
numbers.  Low-precision tensors are drawn in fp32, rounded once to the storage
type, and that rounded tensor is what both the oracle side and the HIP side see.

Small tensors (CTC logits, ids, lengths) come from numpy PCG64 streams; large
tensors (decoder weights, speech embeddings) come from torch generators so they
can be drawn directly on an accelerator and copied back for the oracle.
"""
import math
from dataclasses import dataclass
from typing import List, Optional

import numpy as np
import torch

from .configs import ModelCfg, Workload

_TORCH_DTYPE = {"bf16": torch.bfloat16, "f32": torch.float32}


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, stream]))


@dataclass
class CtcBatch:
    logits: torch.Tensor          # [sum_T, V_ctc], storage dtype of the workload, CPU
    cu_frames: np.ndarray         # int32 [B+1]
    seconds: np.ndarray           # float64 [B]
    confident: np.ndarray         # bool [B]: planted to be far below the entropy threshold
    planted_tokens: List[np.ndarray]   # per utterance, CTC ids of the planted transcript
    planted_path: np.ndarray      # int32 [sum_T], planted frame alignment


def _plant_alignment(rng, T: int, U: int, V: int, blank: int):
    """Token ids and a frame alignment: each token held 1-2 frames, blanks fill the rest."""
    U = max(0, min(U, T // 2))
    labels = [v for v in range(V) if v != blank]
    toks = rng.choice(labels, size=U) if U else np.zeros(0, dtype=np.int64)
    dur = rng.integers(1, 3, size=U)
    while dur.sum() > T:
        dur[int(rng.integers(0, U))] = 1
    n_blank = T - int(dur.sum())
    gaps = rng.multinomial(n_blank, np.full(U + 1, 1.0 / (U + 1)))
    # equal neighbours are only legal when a blank separates them
    for i in range(1, U):
        if gaps[i] == 0 and toks[i] == toks[i - 1]:
            toks[i] = labels[(labels.index(int(toks[i])) + 1) % len(labels)]
    path = []
    for i in range(U):
        path += [blank] * int(gaps[i]) + [int(toks[i])] * int(dur[i])
    path += [blank] * int(gaps[U])
    assert len(path) == T
    return toks.astype(np.int32), np.asarray(path, dtype=np.int32)


def make_ctc_batch(wl: Workload, seed: Optional[int] = None) -> CtcBatch:
    seed = wl.seed if seed is None else seed
    r_len, r_tok, r_noise = _rng(seed, 1), _rng(seed, 2), _rng(seed, 3)
    lo, hi = wl.seconds
    seconds = r_len.uniform(lo, hi, size=wl.B) if hi > lo else np.full(wl.B, lo)
    T = np.maximum(1, np.rint(seconds * wl.frames_per_s).astype(np.int64))
    n_conf = int(round(wl.gate_rate * wl.B))
    confident = np.zeros(wl.B, dtype=bool)
    if n_conf:
        confident[r_len.choice(wl.B, size=n_conf, replace=False)] = True
    cu = np.zeros(wl.B + 1, dtype=np.int32)
    cu[1:] = np.cumsum(T)
    z = r_noise.standard_normal((int(cu[-1]), wl.V_ctc), dtype=np.float32)
    toks_all, path_all = [], np.empty(int(cu[-1]), dtype=np.int32)
    for b in range(wl.B):
        if wl.draft_tokens[0] >= 0:
            U = int(r_tok.integers(wl.draft_tokens[0], wl.draft_tokens[1] + 1))
        else:
            U = int(round(wl.draft_per_s * seconds[b]))
        toks, path = _plant_alignment(r_tok, int(T[b]), U, wl.V_ctc, wl.blank_id)
        toks_all.append(toks)
        path_all[cu[b]:cu[b + 1]] = path
        rows = np.arange(cu[b], cu[b + 1])
        if confident[b]:
            boost = np.full(len(rows), 16.0, dtype=np.float32)
        else:
            boost = np.where(r_noise.random(len(rows)) < 0.6, 8.0, 5.0).astype(np.float32)
        z[rows, path] += boost
    logits = torch.from_numpy(z).to(_TORCH_DTYPE[wl.model.dtype])
    return CtcBatch(logits, cu, seconds, confident, toks_all, path_all)


@dataclass
class CtcHeadBatch:
    enc_h: torch.Tensor           # [sum_T, d_enc] encoder output states, storage dtype, CPU
    w_ctc: torch.Tensor           # [V_ctc, d_enc] output-layer weight, storage dtype
    bias: torch.Tensor            # [V_ctc] fp32
    cu_frames: np.ndarray         # int32 [B+1]
    confident: np.ndarray         # bool [B]
    planted_path: np.ndarray      # int32 [sum_T]


def make_ctc_head_batch(wl: Workload, d_enc: int = 1024, V_ctc: Optional[int] = None,
                        seed: Optional[int] = None) -> CtcHeadBatch:
    """Encoder states and an output layer whose logits look like make_ctc_batch's.

    W rows are N(0, 1/d_enc) (unit norm on average), bias N(0, 0.1^2).  A frame's state is unit
    Gaussian noise plus boost * W[y] / |W[y]|^2 for its planted symbol y, so its logits are ~N(0,1)
    noise with the planted symbol raised by `boost` (16 for confident utterances, 8 or 5 otherwise).
    """
    seed = wl.seed if seed is None else seed
    V = wl.V_ctc if V_ctc is None else V_ctc
    r_len, r_tok, r_noise, r_w = _rng(seed, 11), _rng(seed, 12), _rng(seed, 13), _rng(seed, 14)
    lo, hi = wl.seconds
    seconds = r_len.uniform(lo, hi, size=wl.B) if hi > lo else np.full(wl.B, lo)
    T = np.maximum(1, np.rint(seconds * wl.frames_per_s).astype(np.int64))
    n_conf = int(round(wl.gate_rate * wl.B))
    confident = np.zeros(wl.B, dtype=bool)
    if n_conf:
        confident[r_len.choice(wl.B, size=n_conf, replace=False)] = True
    cu = np.zeros(wl.B + 1, dtype=np.int32)
    cu[1:] = np.cumsum(T)
    dt = _TORCH_DTYPE[wl.model.dtype]
    w = (r_w.standard_normal((V, d_enc)) / math.sqrt(d_enc)).astype(np.float32)
    w = torch.from_numpy(w).to(dt)
    wf = w.float().numpy()
    unit = wf / (wf * wf).sum(axis=1, keepdims=True)
    bias = torch.from_numpy((0.1 * r_w.standard_normal(V)).astype(np.float32))
    h = r_noise.standard_normal((int(cu[-1]), d_enc), dtype=np.float32)
    path_all = np.empty(int(cu[-1]), dtype=np.int32)
    for b in range(wl.B):
        if wl.draft_tokens[0] >= 0:
            U = int(r_tok.integers(wl.draft_tokens[0], wl.draft_tokens[1] + 1))
        else:
            U = int(round(wl.draft_per_s * seconds[b]))
        _, path = _plant_alignment(r_tok, int(T[b]), U, V, min(wl.blank_id, V - 1))
        path_all[cu[b]:cu[b + 1]] = path
        n = len(path)
        if confident[b]:
            boost = np.full(n, 16.0, dtype=np.float32)
        else:
            boost = np.where(r_noise.random(n) < 0.6, 8.0, 5.0).astype(np.float32)
        h[cu[b]:cu[b + 1]] += boost[:, None] * unit[path]
    return CtcHeadBatch(torch.from_numpy(h).to(dt), w, bias, cu, confident, path_all)


def make_ctc_to_llm_map(wl: Workload, seed: Optional[int] = None) -> np.ndarray:
    """Fixed injective table CTC id -> LLM token id (stands in for re-tokenisation)."""
    seed = wl.seed if seed is None else seed
    return _rng(seed, 4).choice(wl.model.vocab, size=wl.V_ctc, replace=False).astype(np.int32)


def _randn(shape, std, dtype, gen, device, mean=0.0):
    t = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
    t.mul_(std)
    if mean:
        t.add_(mean)
    return t.to(dtype)


def make_model_weights(m: ModelCfg, seed: int, device="cpu") -> dict:
    """Random-init decoder: every matrix N(0, 0.02^2); norm gains 1 + N(0, 0.05^2)."""
    dt = _TORCH_DTYPE[m.dtype]
    gen = torch.Generator(device=device)
    gen.manual_seed(seed * 7919 + 11)
    w = {"embed": _randn((m.vocab, m.d_model), 0.02, dt, gen, device),
         "lm_head": _randn((m.vocab, m.d_model), 0.02, dt, gen, device),
         "norm_final": _randn((m.d_model,), 0.05, dt, gen, device, mean=1.0),
         "layers": []}
    for _ in range(m.n_layers):
        w["layers"].append({
            "wq": _randn((m.d_q, m.d_model), 0.02, dt, gen, device),
            "wk": _randn((m.d_kv, m.d_model), 0.02, dt, gen, device),
            "wv": _randn((m.d_kv, m.d_model), 0.02, dt, gen, device),
            "wo": _randn((m.d_model, m.d_q), 0.02, dt, gen, device),
            "w_gate": _randn((m.d_ff, m.d_model), 0.02, dt, gen, device),
            "w_up": _randn((m.d_ff, m.d_model), 0.02, dt, gen, device),
            "w_down": _randn((m.d_model, m.d_ff), 0.02, dt, gen, device),
            "norm_attn": _randn((m.d_model,), 0.05, dt, gen, device, mean=1.0),
            "norm_mlp": _randn((m.d_model,), 0.05, dt, gen, device, mean=1.0),
        })
    return w


@dataclass
class VerifyInputs:
    speech_emb: torch.Tensor      # [sum_S, d] storage dtype
    cu_speech: np.ndarray         # int32 [Bv+1]
    prompt_ids: np.ndarray        # int32 [sum_P]
    cu_prompt: np.ndarray         # int32 [Bv+1]
    draft_ids: np.ndarray         # int32 [sum_U] LLM token ids
    cu_draft: np.ndarray          # int32 [Bv+1]


def make_verify_inputs(wl: Workload, seconds: np.ndarray, drafts: List[np.ndarray],
                       seed: Optional[int] = None, device="cpu") -> VerifyInputs:
    """Inputs of the verification pass for the given utterances (those that failed the gate).

    `drafts` are LLM token ids per utterance.  `corrupt_frac` of the positions are
    overwritten with uniform random ids.
    """
    seed = wl.seed if seed is None else seed
    m = wl.model
    r = _rng(seed, 5)
    Bv = len(drafts)
    S = [wl.speech_fixed if wl.speech_fixed >= 0 else max(1, int(round(wl.speech_per_s * s)))
         for s in seconds]
    cu_s = np.zeros(Bv + 1, dtype=np.int32); cu_s[1:] = np.cumsum(S)
    cu_p = np.arange(Bv + 1, dtype=np.int32) * wl.prompt_len
    cu_d = np.zeros(Bv + 1, dtype=np.int32); cu_d[1:] = np.cumsum([len(d) for d in drafts])
    prompt = r.integers(0, m.vocab, size=int(cu_p[-1])).astype(np.int32)
    dr = (np.concatenate(drafts) if Bv else np.zeros(0)).astype(np.int32)
    if wl.corrupt_frac > 0 and len(dr):
        hit = r.random(len(dr)) < wl.corrupt_frac
        dr = np.where(hit, r.integers(0, m.vocab, size=len(dr)), dr).astype(np.int32)
    gen = torch.Generator(device=device)
    gen.manual_seed(seed * 7919 + 13)
    emb = _randn((int(cu_s[-1]), m.d_model), 0.02, _TORCH_DTYPE[m.dtype], gen, device)
    return VerifyInputs(emb, cu_s, prompt, cu_p, dr, cu_d)


def make_qformer_weights(seed: int, n_q: int = 3, d_h: int = 1024, d_enc: int = 1024, d_out: int = 2048, device="cpu") -> dict:
    """Weights of the projector's windowed cross-attention, bf16: projected queries N(0,1), key / value
    projections N(0, 1/d_enc), output projection N(0, 1/d_h) (scores and outputs of order one on unit-variance
    encoder states)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(seed * 7919 + 17)
    dt = torch.bfloat16
    return {"q_proj": _randn((n_q, d_h), 1.0, dt, gen, device),
            "w_k": _randn((d_h, d_enc), 1.0 / math.sqrt(d_enc), dt, gen, device),
            "w_v": _randn((d_h, d_enc), 1.0 / math.sqrt(d_enc), dt, gen, device),
            "w_o": _randn((d_out, d_h), 1.0 / math.sqrt(d_h), dt, gen, device)}
