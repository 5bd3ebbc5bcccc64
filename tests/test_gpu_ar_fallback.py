"""GPU parity of the auto-regressive fallback (verify_forward_kv + accept_prefix + ar_fallback) against
the oracle's greedy continuation from the accepted prefix (Sec. 2.3, Eq. 6)."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import ssd_oracle as O
from tests.parity import TOL_LOGP, check_accept_len
from tests.test_gpu_verify import _dev, _gate_drafts, _tau_for
from workloads import WORKLOADS, make_ctc_batch, make_model_weights, make_verify_inputs
from workloads.configs import scaled_down

pytestmark = pytest.mark.gpu


def _run_chain(wl, w, vi, tau, n_steps, operand="f16"):
    """verify (with K/V cache) -> accept (with greedy tokens) -> AR continuation of every utterance."""
    from paper_2603_11243_amd.binding import Context
    ctx = Context(wl.model, w, operand=operand)
    Bv = len(vi.cu_draft) - 1
    S, P, U = np.diff(vi.cu_speech), np.diff(vi.cu_prompt), np.diff(vi.cu_draft)
    n = S + P + U
    cap = n + n_steps + 3
    kv_start = np.concatenate([[0], np.cumsum(cap)[:-1]]).astype(np.int32)
    ctx.set_kv_cache(int(cap.sum()))
    ctx.reserve(max_tokens=int(n.sum()), max_verify_rows=int(U.sum()), max_utts=Bv, ar_utts=Bv, ar_steps=n_steps)
    p_ids, d_ids = _dev(vi.prompt_ids), _dev(vi.draft_ids)
    hv = ctx.verify_forward(vi.speech_emb.cuda(), vi.cu_speech, p_ids, vi.cu_prompt, d_ids, vi.cu_draft, kv_start=kv_start)
    acc = ctx.accept_prefix(hv, d_ids, vi.cu_draft, tau, want_greedy=True)
    torch.cuda.synchronize()
    acc_len = acc["accept_len"].cpu().numpy()
    greedy = acc["greedy_tok"].cpu().numpy()
    # Eq. 7: utterances whose draft is not fully accepted continue from the accepted prefix; the first
    # token is the greedy token at the first rejected position
    rej = np.flatnonzero(acc_len < U)
    first = np.array([greedy[vi.cu_draft[b] + acc_len[b]] for b in rej], dtype=np.int32)
    ctx_len = (S + P + acc_len)[rej].astype(np.int32)
    out = ctx.ar_fallback(kv_start[rej], ctx_len, _dev(first), n_steps)
    torch.cuda.synchronize()
    toks = out.cpu().numpy()                      # [n_steps, Br]
    ctx.close()
    return acc_len, rej, first, toks, acc["draft_logp"].cpu().numpy()


def _check_against_oracle(wl, w, vi, tau, n_steps, acc_len, rej, first, toks, logp_gpu, sample=None, tol=None):
    """sample: positions in `rej` to check (default: every rejected utterance)."""
    from tests.test_gpu_verify import _subset
    tol = TOL_LOGP[wl.model.dtype] if tol is None else tol
    ks = list(range(len(rej))) if sample is None else list(sample)
    sub = _subset(vi, [int(rej[k]) for k in ks])
    lp_sub = O.draft_logp(w, wl.model, sub.speech_emb, sub.cu_speech, sub.prompt_ids, sub.cu_prompt, sub.draft_ids, sub.cu_draft)
    w_lm = w["lm_head"].double().cpu().numpy()
    n_exact = 0
    for j, k in enumerate(ks):
        b = rej[k]
        check_accept_len(acc_len[b], False, lp_sub[j], tau, tol)
        sp = vi.speech_emb[vi.cu_speech[b]:vi.cu_speech[b + 1]]
        pr = vi.prompt_ids[vi.cu_prompt[b]:vi.cu_prompt[b + 1]]
        prefix = vi.draft_ids[vi.cu_draft[b]:vi.cu_draft[b] + acc_len[b]]
        # the oracle continues from the prefix the GPU accepted (the prefix decision has its own check above)
        want = O.ar_fallback(w, wl.model, sp, pr, prefix, n_steps)
        got = np.concatenate([[first[k]], toks[:, k]])
        for t in range(n_steps + 1):
            if got[t] == want[t]:
                n_exact += 1
                continue
            # a different token is only legal where the oracle's two best logits are within tolerance;
            # after that the two continuations condition on different tokens and are not comparable
            ids = np.concatenate([pr, prefix, want[:t]]).astype(np.int64)
            x = np.concatenate([O._f64(sp), O._f64(w["embed"][ids])]) if len(ids) else O._f64(sp)
            hfin = O.rmsnorm(O.decoder_hidden([x], w, wl.model)[0][-1], O._f64(w["norm_final"]), wl.model.rms_eps)
            logits = w_lm @ hfin
            assert logits.max() - logits[got[t]] <= tol, f"utt {b} step {t}: token {got[t]} vs oracle {want[t]}"
            break
    return n_exact


def test_ar_fallback_tiny_f32():
    wl = WORKLOADS["cfg1_tiny_f32"]
    cb = make_ctc_batch(wl)
    fail, drafts = _gate_drafts(wl, cb)
    vi = make_verify_inputs(wl, cb.seconds[fail], drafts)
    w = make_model_weights(wl.model, wl.seed)
    tau = 2.3e-4                      # just below 1/vocab: about half of the random draft tokens fail
    n_steps = 12
    res = _run_chain(wl, w, vi, tau, n_steps)
    assert len(res[1]) >= 2
    n_exact = _check_against_oracle(wl, w, vi, tau, n_steps, *res)
    assert n_exact >= (n_steps + 1) * len(res[1]) // 2


def test_ar_fallback_tiny_f32_sharper_model():
    """Larger weights: peaked distributions, so token choices are far from ties and the whole
    continuation must match."""
    wl = replace(WORKLOADS["cfg1_tiny_f32"], model=replace(WORKLOADS["cfg1_tiny_f32"].model, n_layers=3))
    w = make_model_weights(wl.model, 78)
    g = torch.Generator().manual_seed(6)
    for L in w["layers"]:
        for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
            L[k] = torch.randn(L[k].shape, generator=g) * 0.08
    w["lm_head"] = torch.randn(w["lm_head"].shape, generator=g) * 0.3
    w["embed"] = torch.randn(w["embed"].shape, generator=g) * 0.5
    cb = make_ctc_batch(wl)
    fail, drafts = _gate_drafts(wl, cb)
    vi = make_verify_inputs(wl, cb.seconds[fail], drafts)
    tau = 1e-3
    n_steps = 10
    res = _run_chain(wl, w, vi, tau, n_steps)
    n_exact = _check_against_oracle(wl, w, vi, tau, n_steps, *res)
    assert n_exact == (n_steps + 1) * len(res[1])


# B = 5 / 4: at most 32 rejected utterances, the few-row path (register-streaming projections, K-split QKV finished
# inside the decode attention); B = 48: more than 32 rows per step, the LDS-ring projections with the rotary
# epilogue and the plain decode attention
@pytest.mark.parametrize("name,layers,B,n_steps", [("cfg3_1b_ragged64", 2, 5, 4), ("cfg5_3b_ragged128", 1, 4, 4),
                                                   ("cfg3_1b_ragged64", 1, 48, 2)])
def test_ar_fallback_bf16_reduced_depth(name, layers, B, n_steps):
    wl = replace(scaled_down(WORKLOADS[name], n_layers=layers, B=B), gate_rate=0.0)
    cb = make_ctc_batch(wl)
    fail, drafts = _gate_drafts(wl, cb)
    vi = make_verify_inputs(wl, cb.seconds[fail], drafts, device="cuda")
    w = make_model_weights(wl.model, wl.seed, device="cuda")
    tau = _tau_for(wl)
    res = _run_chain(wl, w, vi, tau, n_steps)
    assert len(res[1]) >= (33 if B > 32 else 1)
    n_exact = _check_against_oracle(wl, w, vi, tau, n_steps, *res)
    print(f"{wl.name}: {n_exact} of {(n_steps + 1) * len(res[1])} generated tokens identical to the oracle's")
    assert n_exact >= (n_steps + 1) * len(res[1]) // 2


@pytest.mark.parametrize("name", ["cfg3_1b_ragged64", "cfg4_1b_long_ml"])
def test_ar_fallback_bf16_full_size_sampled_utterances(name):
    """Full 24-layer 1B-class decoder, whole batch on the GPU: the ragged batch of 64 (contexts up to about 200 rows)
    and the long-form batch (every context beyond 256 rows, so that each wavefront of the decode attention walks more
    than one block of keys).  The oracle continues the rejected utterance with the shortest and the one with the
    longest context."""
    wl = WORKLOADS[name]
    cb = make_ctc_batch(wl)
    fail, drafts = _gate_drafts(wl, cb)
    vi = make_verify_inputs(wl, cb.seconds[fail], drafts, device="cuda")
    w = make_model_weights(wl.model, wl.seed, device="cuda")
    tau = _tau_for(wl)
    n_steps = 2
    res = _run_chain(wl, w, vi, tau, n_steps)
    rej = res[1]
    assert 1 <= len(rej) <= 32                     # the few-row path of the step, as in the benchmark
    ctx_len = (np.diff(vi.cu_speech) + np.diff(vi.cu_prompt))[rej] + res[0][rej]
    by_ctx = np.argsort(ctx_len, kind="stable")
    sample = sorted({int(by_ctx[0]), int(by_ctx[-1])})
    if name == "cfg4_1b_long_ml":
        assert ctx_len[by_ctx[-1]] > 256
    n_exact = _check_against_oracle(wl, w, vi, tau, n_steps, *res, sample=sample)
    print(f"{wl.name}: {n_exact} of {(n_steps + 1) * len(sample)} generated tokens identical to the oracle's")
    assert n_exact >= (n_steps + 1) * len(sample) // 2


def test_ar_fallback_bfloat16_operands():
    """The bfloat16 operand type through the whole chain (K/V cache rows, fused decode attention, few-row
    projections): two 1B-width layers, tokens against the oracle's continuation with the wider tolerance of
    that operand type for near-ties."""
    wl = replace(scaled_down(WORKLOADS["cfg3_1b_ragged64"], n_layers=2, B=5), gate_rate=0.0)
    cb = make_ctc_batch(wl)
    fail, drafts = _gate_drafts(wl, cb)
    vi = make_verify_inputs(wl, cb.seconds[fail], drafts, device="cuda")
    w = make_model_weights(wl.model, wl.seed, device="cuda")
    tau = _tau_for(wl)
    n_steps = 4
    res = _run_chain(wl, w, vi, tau, n_steps, operand="bf16")
    assert len(res[1]) >= 1
    n_exact = _check_against_oracle(wl, w, vi, tau, n_steps, *res, tol=10 * TOL_LOGP["bf16"])
    print(f"{wl.name}, bfloat16 operands: {n_exact} of {(n_steps + 1) * len(res[1])} generated tokens identical to the oracle's")
    assert n_exact >= (n_steps + 1) * len(res[1]) // 2
