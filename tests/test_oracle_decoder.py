"""Pins for the oracle's decoder forward, LM-head scoring and acceptance rule.

The decoder is a textbook composition, so it is pinned to torch CPU float64 library
routines (scaled_dot_product_attention, rms_norm, silu, log_softmax, embedding) wired
together independently here, plus special cases and invariants.
"""
import math
import os
from dataclasses import replace

import numpy as np
import torch
import torch.nn.functional as F

from oracle import ssd_oracle as O
from workloads import configs as C
from workloads import synth

GOLD = {}
with open(os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")) as f:
    for line in f:
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            GOLD[k] = float(v)

SMALL = C.ModelCfg(n_layers=3, d_model=64, n_q_heads=6, n_kv_heads=2, head_dim=16, d_ff=96,
                   vocab=211, dtype="f32", rope_theta=10000.0)


def _weights(cfg, seed=3, std=0.2):
    w = synth.make_model_weights(cfg, seed)
    # larger weights than the workloads' 0.02 so that attention is far from uniform
    g = torch.Generator().manual_seed(seed)
    for L in w["layers"]:
        for k in L:
            if L[k].ndim == 2:
                L[k] = torch.randn(L[k].shape, generator=g) * std
    w["lm_head"] = torch.randn(w["lm_head"].shape, generator=g) * std
    w["embed"] = torch.randn(w["embed"].shape, generator=g)
    return w


def _torch_rope(v, theta):
    # complex form: (v_i + j v_{i+hd/2}) * exp(j * pos * theta^(-2i/hd))
    n, h, hd = v.shape
    half = hd // 2
    inv = torch.pow(torch.tensor(theta, dtype=torch.float64),
                    -2.0 * torch.arange(half, dtype=torch.float64) / hd)
    ang = torch.arange(n, dtype=torch.float64)[:, None] * inv[None, :]
    c = torch.complex(v[..., :half], v[..., half:]) * torch.polar(torch.ones_like(ang), ang)[:, None, :]
    return torch.cat([c.real, c.imag], dim=-1)


def _torch_forward(x, w, cfg):
    """Independent float64 forward from torch library ops; x: [n, d] tensor."""
    n = x.shape[0]
    for L in w["layers"]:
        L = {k: v.double() for k, v in L.items()}
        a = F.rms_norm(x, (cfg.d_model,), L["norm_attn"], cfg.rms_eps)
        q = _torch_rope(F.linear(a, L["wq"]).view(n, cfg.n_q_heads, cfg.head_dim), cfg.rope_theta)
        k = _torch_rope(F.linear(a, L["wk"]).view(n, cfg.n_kv_heads, cfg.head_dim), cfg.rope_theta)
        v = F.linear(a, L["wv"]).view(n, cfg.n_kv_heads, cfg.head_dim)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], is_causal=True, enable_gqa=True)
        x = x + F.linear(o[0].transpose(0, 1).reshape(n, -1), L["wo"])
        b = F.rms_norm(x, (cfg.d_model,), L["norm_mlp"], cfg.rms_eps)
        x = x + F.linear(F.silu(F.linear(b, L["w_gate"])) * F.linear(b, L["w_up"]), L["w_down"])
    return x


def _inputs(cfg, S, P, U, seed=0):
    rng = np.random.default_rng(seed)
    Bv = len(S)
    cu = lambda a: np.concatenate([[0], np.cumsum(a)]).astype(np.int32)
    sp = torch.from_numpy(rng.normal(size=(int(sum(S)), cfg.d_model)))
    return dict(speech_emb=sp, cu_speech=cu(S),
                prompt_ids=rng.integers(0, cfg.vocab, size=int(sum(P))).astype(np.int32), cu_prompt=cu(P),
                draft_ids=rng.integers(0, cfg.vocab, size=int(sum(U))).astype(np.int32), cu_draft=cu(U))


def test_forward_matches_torch_library_ops_gqa():
    cfg = SMALL
    w = _weights(cfg)
    inp = _inputs(cfg, S=[5, 9], P=[3, 2], U=[7, 4])
    got = O.draft_logp(w, cfg, **inp)
    for b in range(2):
        S = inp["cu_speech"][b + 1] - inp["cu_speech"][b]; P = inp["cu_prompt"][b + 1] - inp["cu_prompt"][b]
        pid = torch.from_numpy(inp["prompt_ids"][inp["cu_prompt"][b]:inp["cu_prompt"][b + 1]]).long()
        did = torch.from_numpy(inp["draft_ids"][inp["cu_draft"][b]:inp["cu_draft"][b + 1]]).long()
        x = torch.cat([inp["speech_emb"][inp["cu_speech"][b]:inp["cu_speech"][b + 1]],
                       F.embedding(pid, w["embed"].double()), F.embedding(did, w["embed"].double())])
        h = _torch_forward(x, w, cfg)
        hn = F.rms_norm(h, (cfg.d_model,), w["norm_final"].double(), cfg.rms_eps)
        lsm = F.log_softmax(F.linear(hn, w["lm_head"].double()), dim=-1)
        U = len(did)
        want = lsm[S + P - 1: S + P - 1 + U].gather(1, did[:, None])[:, 0].numpy()
        assert np.allclose(got[b], want, rtol=0, atol=1e-10)
        assert np.abs(want).max() > 1.0       # non-trivial distribution


def test_forward_matches_torch_library_ops_mha_tiny_shape():
    cfg = replace(C.TINY, n_layers=2, vocab=512)
    w = _weights(cfg, std=0.08)
    inp = _inputs(cfg, S=[30], P=[10], U=[12], seed=4)
    got = O.draft_logp(w, cfg, **inp)[0]
    pid = torch.from_numpy(inp["prompt_ids"]).long(); did = torch.from_numpy(inp["draft_ids"]).long()
    x = torch.cat([inp["speech_emb"], F.embedding(pid, w["embed"].double()), F.embedding(did, w["embed"].double())])
    hn = F.rms_norm(_torch_forward(x, w, cfg), (cfg.d_model,), w["norm_final"].double(), cfg.rms_eps)
    lsm = F.log_softmax(F.linear(hn, w["lm_head"].double()), dim=-1)
    want = lsm[39:39 + 12].gather(1, did[:, None])[:, 0].numpy()
    assert np.allclose(got, want, rtol=0, atol=1e-10)


def test_rope_properties():
    rng = np.random.default_rng(5)
    v = rng.normal(size=(9, 2, 16)); pos = np.arange(9)
    r = O.rope(v, pos, 10000.0)
    assert np.allclose(r[0], v[0])                                      # position 0: identity
    assert np.allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(v, axis=-1))
    # q_m . k_n depends on m - n only
    q = np.tile(rng.normal(size=(1, 1, 16)), (9, 1, 1)); k = np.tile(rng.normal(size=(1, 1, 16)), (9, 1, 1))
    rq, rk = O.rope(q, pos, 10000.0), O.rope(k, pos, 10000.0)
    assert np.allclose(rq[5, 0] @ rk[3, 0], rq[8, 0] @ rk[6, 0])
    assert not np.allclose(rq[5, 0] @ rk[3, 0], rq[5, 0] @ rk[4, 0])
    # the first pair (i = 0) turns by exactly `pos` radians, the pairing is (i, i + hd/2)
    e = np.zeros((4, 1, 16)); e[:, 0, 0] = 1.0
    re = O.rope(e, np.arange(4), 10000.0)
    assert np.allclose(re[:, 0, 0], np.cos(np.arange(4))) and np.allclose(re[:, 0, 8], np.sin(np.arange(4)))
    # last pair turns by pos * theta^(-(hd-2)/hd)
    e = np.zeros((2, 1, 16)); e[:, 0, 7] = 1.0
    re = O.rope(e, np.array([0, 3]), 10000.0)
    assert np.allclose(re[1, 0, 15], math.sin(3 * 10000.0 ** (-14 / 16)))


def test_rmsnorm_scale_invariance_and_unit_rms():
    rng = np.random.default_rng(6)
    x = rng.normal(size=(4, 32)); w = rng.normal(size=32)
    a = O.rmsnorm(x, w, 0.0)
    assert np.allclose(O.rmsnorm(7.0 * x, w, 0.0), a)
    assert np.allclose(np.sqrt(np.mean(O.rmsnorm(x, np.ones(32), 0.0) ** 2, axis=-1)), 1.0)
    assert np.allclose(O.rmsnorm(np.full((1, 32), 2.0), w, 5.0), 2.0 / 3.0 * w)     # eps is added to mean(x^2)


def test_layer_special_cases():
    cfg = SMALL
    w = _weights(cfg)
    L = {k: v.double().numpy() for k, v in w["layers"][0].items()}
    rng = np.random.default_rng(7)
    x = rng.normal(size=(6, cfg.d_model))
    # zero output projections: the layer is the identity
    Lz = dict(L, wo=np.zeros_like(L["wo"]), w_down=np.zeros_like(L["w_down"]))
    assert np.array_equal(O.decoder_layer(x, Lz, cfg), x)
    # a single position attends only to itself: attention output is its own v, for each query head's KV group
    Lm = dict(L, w_down=np.zeros_like(L["w_down"]))
    x1 = x[:1]
    a = O.rmsnorm(x1, L["norm_attn"], cfg.rms_eps)
    v = (a @ L["wv"].T).reshape(cfg.n_kv_heads, cfg.head_dim)
    o = np.concatenate([v[h // (cfg.n_q_heads // cfg.n_kv_heads)] for h in range(cfg.n_q_heads)])
    assert np.allclose(O.decoder_layer(x1, Lm, cfg), x1 + o @ L["wo"].T)
    # the first position of a longer sequence gives the same output (causal mask)
    assert np.allclose(O.decoder_layer(x, L, cfg)[0], O.decoder_layer(x1, L, cfg)[0])


def test_causality_and_prefix_consistency():
    cfg = SMALL
    w = _weights(cfg)
    inp = _inputs(cfg, S=[6], P=[3], U=[8], seed=8)
    base = O.draft_logp(w, cfg, **inp)[0]
    k = 5                                          # change draft token k (1-based): logp_i for i < k unchanged
    inp2 = dict(inp, draft_ids=inp["draft_ids"].copy())
    inp2["draft_ids"][k - 1] = (inp2["draft_ids"][k - 1] + 1) % cfg.vocab
    mod = O.draft_logp(w, cfg, **inp2)[0]
    assert np.allclose(mod[:k - 1], base[:k - 1], atol=1e-13)
    assert not np.isclose(mod[k - 1], base[k - 1]) and not np.isclose(mod[k], base[k])
    # truncating the draft leaves the scores of the kept tokens unchanged
    inp3 = dict(inp, draft_ids=inp["draft_ids"][:4], cu_draft=np.array([0, 4], np.int32))
    assert np.allclose(O.draft_logp(w, cfg, **inp3)[0], base[:4], atol=1e-13)


def test_lm_head_normalisation_and_gather():
    cfg = SMALL
    w = _weights(cfg)
    inp = _inputs(cfg, S=[4], P=[2], U=[3], seed=9)
    lp, hid, greedy = O.draft_logp(w, cfg, return_hidden=True, return_greedy=True, **inp)
    W = w["lm_head"].double().numpy()
    for i in range(3):
        # brute force over the whole vocabulary: scoring each candidate token in turn sums to one
        logits = W @ hid[0][i]
        p = np.exp(logits - logits.max()); p /= p.sum()
        assert abs(p.sum() - 1) < 1e-12 and lp[0][i] <= 0
        assert abs(math.exp(lp[0][i]) - p[inp["draft_ids"][i]]) < 1e-12
        assert greedy[0][i] == int(np.argmax(p))
    # one-hot LM head rows: logit of token v is coordinate v of the normed hidden row
    w2 = dict(w, lm_head=torch.eye(cfg.vocab, cfg.d_model))
    lp2, hid2 = O.draft_logp(w2, cfg, return_hidden=True, **dict(inp, draft_ids=np.array([0, 17, 63], np.int32)))
    for i, tok in enumerate([0, 17, 63]):
        logits = np.concatenate([hid2[0][i], np.zeros(cfg.vocab - cfg.d_model)])
        want = logits[tok] - math.log(np.exp(logits).sum())
        assert abs(lp2[0][i] - want) < 1e-12


def test_lm_head_logp_closed_forms():
    """The Eq. 5 step at one position, on its own: cases with a known answer."""
    V, d = 37, 8
    h = np.arange(1, d + 1, dtype=np.float64)
    # all-zero head: the uniform distribution, and the lowest index wins the tie
    lp, g = O.lm_head_logp(h, np.zeros((V, d)), 5)
    assert abs(lp + math.log(V)) < 1e-12 and g == 0
    # one row scaled so that its logit is L, all other logits 0: p = e^L / (e^L + V - 1)
    W = np.zeros((V, d)); W[11] = h / (h @ h) * 3.0
    lp, g = O.lm_head_logp(h, W, 11)
    assert abs(lp - (3.0 - math.log(math.exp(3.0) + V - 1))) < 1e-12 and g == 11
    lp_other, _ = O.lm_head_logp(h, W, 4)
    assert abs(lp_other - (0.0 - math.log(math.exp(3.0) + V - 1))) < 1e-12
    # shifting every logit by a constant (a bias direction in h) changes nothing; huge logits do not overflow
    rng = np.random.default_rng(0)
    W = rng.normal(size=(V, d))
    base = [O.lm_head_logp(h, W, t)[0] for t in range(V)]
    assert abs(sum(math.exp(x) for x in base) - 1) < 1e-12
    big = [O.lm_head_logp(h * 1e3, W, t)[0] for t in range(V)]
    assert all(np.isfinite(big)) and abs(max(big)) < 1e-9          # one token takes all the mass
    # two equal maxima: the lowest index is the greedy token
    W2 = W.copy(); W2[20] = W2[3]
    top = int(np.argmax(W2 @ h))
    if top in (3, 20):
        assert O.lm_head_logp(h, W2, 0)[1] == 3


def test_ar_fallback_is_consistent_with_teacher_forced_scoring():
    """Feeding the generated tokens back as a draft: the greedy token at every scoring position is the
    token that was generated there (ties aside, none here), and the first token is the greedy choice
    after the prefix.  This ties the AR loop to the scoring function pinned above."""
    cfg = SMALL
    w = _weights(cfg)
    inp = _inputs(cfg, S=[5], P=[3], U=[4], seed=11)
    toks = O.ar_fallback(w, cfg, inp["speech_emb"], inp["prompt_ids"], inp["draft_ids"][:2], n_steps=5)
    assert len(toks) == 6
    draft = np.concatenate([inp["draft_ids"][:2], toks]).astype(np.int32)
    _, greedy = O.draft_logp(w, cfg, inp["speech_emb"], inp["cu_speech"], inp["prompt_ids"], inp["cu_prompt"], draft,
                             np.array([0, len(draft)], np.int32), return_greedy=True)
    # row i (0-based) scores draft token i: rows 2.. score the generated tokens
    assert list(greedy[0][2:]) == list(toks)
    # an empty prefix and zero steps
    t0 = O.ar_fallback(w, cfg, inp["speech_emb"], inp["prompt_ids"], [], n_steps=0)
    _, g0 = O.draft_logp(w, cfg, inp["speech_emb"], inp["cu_speech"], inp["prompt_ids"], inp["cu_prompt"],
                         np.array([1], np.int32), np.array([0, 1], np.int32), return_greedy=True)
    assert t0[0] == g0[0][0]
    # the continuation does not depend on what the rejected draft tokens were: only the prefix matters
    toks2 = O.ar_fallback(w, cfg, inp["speech_emb"], inp["prompt_ids"], inp["draft_ids"][:2], n_steps=5)
    assert np.array_equal(toks, toks2)


def test_accept_prefix_hand_cases_with_paper_thresholds():
    ln = math.log
    for tau in (GOLD["tau_slm_high_rtfx"], GOLD["tau_slm_high_accuracy"]):
        ok, bad = ln(tau * 1.5), ln(tau * 0.5)
        assert O.accept_prefix([ok, ok, ok], tau) == {"accept_len": 3, "all_accepted": True}
        assert O.accept_prefix([bad, ok, ok], tau) == {"accept_len": 0, "all_accepted": False}
        assert O.accept_prefix([ok, bad, ok], tau) == {"accept_len": 1, "all_accepted": False}
        assert O.accept_prefix([ok, ok, bad], tau) == {"accept_len": 2, "all_accepted": False}
        assert O.accept_prefix([ok, bad, bad, ok], tau)["accept_len"] == 1          # first failure counts
        assert O.accept_prefix([ok, ln(tau), ok], tau)["accept_len"] == 1           # equality fails (strict >)
        assert O.accept_prefix([], tau) == {"accept_len": 0, "all_accepted": True}  # vacuous
    # p = 0.15 passes tau = 0.1 and fails tau = 0.2
    assert O.accept_prefix([ln(0.15)], 0.1)["all_accepted"] and not O.accept_prefix([ln(0.15)], 0.2)["all_accepted"]
    assert O.accept_prefix([-50.0, -60.0], 0.0)["accept_len"] == 2                  # tau <= 0 accepts all
    assert O.accept_prefix([-1e-9], 1.0)["accept_len"] == 0                         # tau >= 1 accepts none


def test_accept_prefix_properties():
    rng = np.random.default_rng(10)
    for _ in range(200):
        U = int(rng.integers(0, 12))
        lp = -rng.exponential(2.0, size=U)
        taus = np.sort(rng.uniform(0.01, 0.9, size=6))
        lens = [O.accept_prefix(lp, t)["accept_len"] for t in taus]
        assert all(a >= b for a, b in zip(lens, lens[1:]))                          # non-increasing in tau
        for t, n in zip(taus, lens):
            brute = next((i for i in range(U) if math.exp(lp[i]) <= t), U)
            assert n == brute
            assert (n == U) == (U == 0 or lp.min() > math.log(t))
            for k in range(n + 1):                                                   # truncation at k <= n
                assert O.accept_prefix(lp[:k], t)["accept_len"] == k


def test_final_hypothesis_case_split():
    assert O.final_hypothesis_case(True, False) == "draft"
    assert O.final_hypothesis_case(False, True) == "draft"
    assert O.final_hypothesis_case(True, True) == "draft"
    assert O.final_hypothesis_case(False, False) == "prefix+ar"


def test_threshold_grid_matches_single_thresholds_and_is_monotone():
    rng = np.random.default_rng(12)
    H = rng.uniform(0.0, 5.0, size=9)
    H[3] = GOLD["tau_ctc_high_accuracy"]                      # equality at a grid point must fail
    lps = [-rng.exponential(1.5, size=int(rng.integers(0, 9))) for _ in range(7)]
    tc = [GOLD["tau_ctc_high_accuracy"], 1.5, GOLD["tau_ctc_high_rtfx"]]
    ts = [GOLD["tau_slm_high_rtfx"], GOLD["tau_slm_high_accuracy"]]
    g = O.threshold_grid(H, lps, tc, ts)
    assert g["gate_pass"].shape == (3, 9) and g["accept_len"].shape == (2, 7)
    assert not g["gate_pass"][0, 3] and g["gate_pass"][1, 3]
    for a, t in enumerate(tc):
        assert list(g["gate_pass"][a]) == [h < t for h in H]
    assert (g["gate_pass"][0] <= g["gate_pass"][2]).all()                      # a looser gate accepts more
    assert (g["accept_len"][0] >= g["accept_len"][1]).all()                    # a stricter likelihood accepts less
    for b, lp in enumerate(lps):
        for a, t in enumerate(ts):
            assert g["accept_len"][a, b] == next((i for i in range(len(lp)) if math.exp(lp[i]) <= t), len(lp))


def test_plan_batches_properties_and_brute_force():
    rng = np.random.default_rng(13)
    for padded in (False, True):
        for _ in range(50):
            n = int(rng.integers(1, 12))
            L = rng.integers(1, 40, size=n)
            budget = int(rng.integers(10, 120))
            bs = O.plan_batches(L, budget, padded)
            flat = [i for b in bs for i in b]
            assert sorted(flat) == list(range(n))                               # a partition
            assert [L[i] for i in flat] == sorted(L, reverse=True)              # longest first
            cost = lambda b: len(b) * max(L[i] for i in b) if padded else sum(L[i] for i in b)
            for k, b in enumerate(bs):
                assert cost(b) <= budget or len(b) == 1
                if k + 1 < len(bs):                                             # greedy: the next utterance did not fit
                    assert cost(b + [bs[k + 1][0]]) > budget
    # the paper's setting: a 50K budget swallows a small sorted batch whole
    assert O.plan_batches([300, 100, 200], 50000, False) == [[0, 2, 1]]
    assert O.plan_batches([30, 10, 20], 45, True) == [[0], [2, 1]]
