"""Pins for the oracle's gate functions (entropy, greedy path, collapse, decision).

Every expected value here comes from a closed form, a library routine, an invariant or
brute force -- never from the oracle itself and never from the HIP path.
"""
import itertools
import math
import os

import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import ssd_oracle as O

GOLD = {}
with open(os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")) as f:
    for line in f:
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            GOLD[k] = float(v)


@pytest.mark.parametrize("V", [256, 348, 512, 2048])
def test_entropy_uniform_is_ln_v(V):
    H = O.frame_entropy(np.full((3, V), 1.2345))
    assert np.allclose(H, GOLD[f"ln_{V}"], rtol=0, atol=1e-12)


def test_entropy_one_hot_is_zero():
    z = np.full((2, 348), -np.inf)
    z[0, 5] = 3.0
    z[1, 347] = -7.0
    assert np.array_equal(O.frame_entropy(z), np.zeros(2))


@pytest.mark.parametrize("V,c", [(256, 8.0), (512, 5.0), (2048, 16.0), (348, -3.0)])
def test_entropy_one_peak_closed_form(V, c):
    # one logit c, the rest 0:  H = ln(e^c + V - 1) - c e^c / (e^c + V - 1)
    z = np.zeros((1, V)); z[0, V // 3] = c
    s = math.exp(c) + V - 1
    want = math.log(s) - c * math.exp(c) / s
    assert abs(O.frame_entropy(z)[0] - want) < 1e-12


def test_entropy_two_point_closed_form():
    # two finite logits a, b (others -inf): binary entropy of sigmoid(a - b)
    z = np.full((1, 16), -np.inf); z[0, 2] = 0.3; z[0, 9] = -1.1
    p = 1.0 / (1.0 + math.exp(-1.4))
    want = -(p * math.log(p) + (1 - p) * math.log(1 - p))
    assert abs(O.frame_entropy(z)[0] - want) < 1e-14


def test_entropy_matches_scipy_and_invariants():
    rng = np.random.default_rng(0)
    z = rng.normal(size=(50, 348)) * 3
    H = O.frame_entropy(z)
    want = scipy.stats.entropy(scipy.special.softmax(z, axis=1), axis=1)
    assert np.allclose(H, want, atol=1e-12)
    assert np.allclose(O.frame_entropy(z + 17.5), H, atol=1e-12)          # shift invariance
    perm = rng.permutation(348)
    assert np.allclose(O.frame_entropy(z[:, perm]), H, atol=1e-12)        # permutation
    assert (H >= 0).all() and (H <= GOLD["ln_348"] + 1e-12).all()
    # a sharper distribution has lower entropy
    assert (O.frame_entropy(2 * z) < H).all()


def test_entropy_rejects_nan_and_plus_inf():
    z = np.zeros((1, 4)); z[0, 1] = np.nan
    with pytest.raises(ValueError):
        O.frame_entropy(z)
    z[0, 1] = np.inf
    with pytest.raises(ValueError):
        O.greedy_alignment(z)


def test_argmax_brute_force_and_ties():
    rng = np.random.default_rng(1)
    z = np.round(rng.normal(size=(200, 37)), 1)      # coarse values: many exact ties
    got = O.greedy_alignment(z)
    for t in range(z.shape[0]):
        best = 0
        for a in range(1, z.shape[1]):
            if z[t, a] > z[t, best]:
                best = a
        assert got[t] == best
    z = np.zeros((1, 10)); z[0, 3] = z[0, 7] = 2.0
    assert O.greedy_alignment(z)[0] == 3
    z = np.array([[-0.0, 0.0, -1.0]])                # signed zeros compare equal
    assert O.greedy_alignment(z)[0] == 0


def test_collapse_hand_paths():
    e, a, b = 0, 5, 9
    assert list(O.collapse([a, a, e, a, b, b, e], e)) == [a, a, b]
    assert list(O.collapse([e, e, e], e)) == []
    assert list(O.collapse([], e)) == []
    assert list(O.collapse([e, a, e, e, b, e], e)) == [a, b]
    assert list(O.collapse([a, b, a, b], e)) == [a, b, a, b]
    assert list(O.collapse([a, a, a], e)) == [a]
    # order matters: duplicates are merged before blanks are dropped, so a blank separates repeats
    assert list(O.collapse([a, e, a], e)) == [a, a]
    # blank need not be id 0
    assert list(O.collapse([3, 7, 7, 3, 3, 7], 7)) == [3, 3]


def test_collapse_all_short_paths_against_groupby_and_streaming():
    blank = 0
    for n in range(0, 9):
        for path in itertools.product((0, 1, 2), repeat=n):
            want = [k for k, _ in itertools.groupby(path) if k != blank]
            got = list(O.collapse(path, blank))
            assert got == want
            assert list(O.collapse_streaming(path, blank)) == want
            assert list(O.collapse(got, blank)) == [k for k, _ in itertools.groupby(got)]
            runs = len([1 for _ in itertools.groupby(path)])
            assert len(got) <= runs


def test_gate_strictness_and_monotonicity():
    V = 348
    z = np.zeros((4, V))                      # uniform frames: H = ln V exactly representable path
    cu = [0, 4]
    H = O.frame_entropy(z)[0]
    assert not O.ctc_gate(z, cu, 0, H)["gate_pass"][0]                 # equality fails (strict <)
    assert O.ctc_gate(z, cu, 0, np.nextafter(H, 10))["gate_pass"][0]
    # paper thresholds: uniform frames fail both, sharply peaked frames pass both
    for tau in (GOLD["tau_ctc_high_accuracy"], GOLD["tau_ctc_high_rtfx"]):
        assert not O.ctc_gate(z, cu, 0, tau)["gate_pass"][0]
        zp = z.copy(); zp[:, 3] = 20.0
        assert O.ctc_gate(zp, cu, 0, tau)["gate_pass"][0]
    # one bad frame is enough to fail the whole utterance; neighbours are unaffected
    zp = np.zeros((6, V)); zp[:, 3] = 20.0; zp[4, 3] = 0.0
    r = O.ctc_gate(zp, [0, 3, 6], 0, 0.7)
    assert list(r["gate_pass"]) == [True, False]
    assert abs(r["max_entropy"][1] - GOLD["ln_348"]) < 1e-12
    # monotone in tau
    rng = np.random.default_rng(2)
    zz = rng.normal(size=(40, 64)) * 4
    prev = False
    for tau in np.linspace(0.1, 4.2, 30):
        cur = bool(O.ctc_gate(zz, [0, 40], 0, tau)["gate_pass"][0])
        assert cur or not prev
        prev = cur


def test_gate_draft_is_collapse_of_argmax_per_utterance():
    V, blank = 12, 0
    path = [0, 4, 4, 0, 4, 7, 7, 0,   3, 3, 3, 0, 0, 3]
    z = np.zeros((len(path), V))
    z[np.arange(len(path)), path] = 9.0
    r = O.ctc_gate(z, [0, 8, 14], blank, 0.7)
    assert [list(d) for d in r["drafts"]] == [[4, 4, 7], [3, 3]]
    assert list(r["frame_argmax"]) == path
    with pytest.raises(ValueError):
        O.ctc_gate(z, [0, 0, 14], blank, 0.7)
