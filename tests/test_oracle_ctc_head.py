"""Pins for the oracle of the CTC output layer fused with the gate.

Expected values come from closed forms, brute force in exact rational arithmetic and special
cases that reduce to the already pinned gate functions -- never from the oracle's own matrix
product and never from the HIP path.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import ssd_oracle as O
from workloads import configs, synth


def test_logits_brute_force_exact_rationals():
    # small integers / dyadic fractions: the float64 result must be exact
    rng = np.random.default_rng(3)
    h = rng.integers(-8, 9, size=(5, 7)) / 4.0
    w = rng.integers(-8, 9, size=(6, 7)) / 8.0
    b = rng.integers(-8, 9, size=6) / 2.0
    z = O.ctc_head_logits(h, w, b)
    assert z.shape == (5, 6)
    for t in range(5):
        for v in range(6):
            want = sum(Fraction(float(h[t, k])) * Fraction(float(w[v, k])) for k in range(7)) + Fraction(float(b[v]))
            assert Fraction(float(z[t, v])) == want        # a transposed operand or a dropped bias fails here


def test_identity_layer_reduces_to_plain_gate():
    # W = I, b = 0: the fused path is the gate on the states themselves
    rng = np.random.default_rng(5)
    V = 12
    h = rng.standard_normal((9, V)) * 3
    cu = [0, 4, 9]
    got = O.ctc_head_gate(h, np.eye(V), None, cu, blank=0, tau_ctc=1.0)
    want = O.ctc_gate(h, cu, 0, 1.0)
    for k in want:
        if isinstance(want[k], list):
            assert all(np.array_equal(a, b) for a, b in zip(got[k], want[k]))
        else:
            assert np.array_equal(got[k], want[k])


def test_zero_weight_gives_bias_distribution():
    # W = 0: every frame has the distribution softmax(b); one-peak closed form for its entropy
    V, c = 348, 6.0
    b = np.zeros(V)
    b[17] = c
    h = np.random.default_rng(7).standard_normal((4, 32))
    res = O.ctc_head_gate(h, np.zeros((V, 32)), b, [0, 4], blank=0, tau_ctc=3.0)
    Z = np.exp(c) + V - 1
    H = np.log(Z) - c * np.exp(c) / Z
    assert np.allclose(res["frame_entropy"], H, rtol=0, atol=1e-12)
    assert np.array_equal(res["frame_argmax"], np.full(4, 17))
    assert [list(d) for d in res["drafts"]] == [[17]]      # four equal frames collapse to one symbol


def test_bias_shift_invariance_and_permutation():
    rng = np.random.default_rng(11)
    h, w, b = rng.standard_normal((6, 16)), rng.standard_normal((10, 16)), rng.standard_normal(10)
    base = O.ctc_head_gate(h, w, b, [0, 6], 0, 1.5)
    shifted = O.ctc_head_gate(h, w, b + 2.5, [0, 6], 0, 1.5)        # softmax ignores a constant
    assert np.allclose(base["frame_entropy"], shifted["frame_entropy"], rtol=0, atol=1e-12)
    assert np.array_equal(base["frame_argmax"], shifted["frame_argmax"])
    perm = rng.permutation(10)
    moved = O.ctc_head_gate(h, w[perm], b[perm], [0, 6], 0, 1.5)    # rows of W are the symbols
    assert np.allclose(base["frame_entropy"], moved["frame_entropy"], rtol=0, atol=1e-12)
    assert np.array_equal(perm[moved["frame_argmax"]], base["frame_argmax"])


def test_bf16_inputs_are_widened_exactly():
    h = torch.tensor([[1.0, 2.0 ** -9, -3.0]], dtype=torch.bfloat16)
    w = torch.tensor([[2.0 ** 7, 1.0, 0.5]], dtype=torch.bfloat16)
    assert O.ctc_head_logits(h, w)[0, 0] == 128.0 + 2.0 ** -9 - 1.5


@pytest.mark.parametrize("name", ["cfg1_tiny_f32", "cfg2_1b_b1"])
def test_synthetic_head_batch_follows_its_recipe(name):
    wl = configs.WORKLOADS[name]
    hb = synth.make_ctc_head_batch(wl, d_enc=256, V_ctc=348 if name != "cfg1_tiny_f32" else None)
    V = hb.w_ctc.shape[0]
    assert hb.enc_h.shape == (hb.cu_frames[-1], 256) and hb.bias.shape == (V,)
    res = O.ctc_head_gate(hb.enc_h, hb.w_ctc, hb.bias, hb.cu_frames, min(wl.blank_id, V - 1), wl.tau_ctc)
    # boosts of +5 and more over unit noise: the planted path is the greedy path on nearly every frame
    assert (res["frame_argmax"] == hb.planted_path).mean() > 0.9
    again = synth.make_ctc_head_batch(wl, d_enc=256, V_ctc=348 if name != "cfg1_tiny_f32" else None)
    assert torch.equal(again.enc_h, hb.enc_h) and torch.equal(again.w_ctc, hb.w_ctc)
