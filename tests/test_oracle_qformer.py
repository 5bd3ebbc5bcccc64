"""Pins for the oracle of the projector's windowed cross-attention (Sec. 3.1: 15 frames -> 3 queries).

Expected values come from a torch-library attention on window-sliced inputs, closed forms and invariants,
never from the oracle's own code and never from the HIP path."""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import ssd_oracle as O


def _params(rng, n_q=3, d_h=32, d_enc=24, d_out=20):
    return (rng.standard_normal((n_q, d_h)), rng.standard_normal((d_h, d_enc)) / np.sqrt(d_enc),
            rng.standard_normal((d_h, d_enc)) / np.sqrt(d_enc), rng.standard_normal((d_out, d_h)) / np.sqrt(d_h))


def test_against_torch_attention_on_window_slices():
    """Independent route: torch's scaled_dot_product_attention (float64) on each window, heads split by view."""
    rng = np.random.default_rng(1)
    n_heads, window = 4, 15
    Q, Wk, Wv, Wo = _params(rng)
    cu = [0, 31, 46, 53]                       # 31 = 15 + 15 + 1, 15 exactly, 7 (one short window)
    Hs = rng.standard_normal((cu[-1], 24)) * 2
    g, cu_s = O.qformer_window_pool(Hs, cu, Q, Wk, Wv, Wo, n_heads, window)
    assert cu_s.tolist() == [0, 9, 12, 15] and g.shape == (15, 20)
    tq, tk, tv, to, th = (torch.from_numpy(a) for a in (Q, Wk, Wv, Wo, Hs))
    row = 0
    for b in range(3):
        for w0 in range(cu[b], cu[b + 1], window):
            hw = th[w0:min(w0 + window, cu[b + 1])]
            n = hw.shape[0]
            k = (hw @ tk.T).view(n, n_heads, -1).transpose(0, 1)            # [heads, n, dh]
            v = (hw @ tv.T).view(n, n_heads, -1).transpose(0, 1)
            q = tq.view(3, n_heads, -1).transpose(0, 1)                     # [heads, 3, dh]
            o = F.scaled_dot_product_attention(q, k, v)                     # default scale 1/sqrt(dh), no mask
            want = o.transpose(0, 1).reshape(3, -1) @ to.T
            assert np.abs(g[row:row + 3] - want.numpy()).max() < 1e-12
            row += 3
    assert row == 15


def test_closed_forms():
    rng = np.random.default_rng(2)
    Q, Wk, Wv, Wo = _params(rng)
    Hs = rng.standard_normal((15, 24))
    # zero queries: uniform attention, every query returns the projected mean of the window
    g, _ = O.qformer_window_pool(Hs, [0, 15], np.zeros_like(Q), Wk, Wv, Wo, 4)
    want = Wo @ (Wv @ Hs.mean(axis=0))
    assert np.abs(g - want[None, :]).max() < 1e-12
    # a window of one frame: softmax over one key is 1, the output is w_o w_v h whatever the query
    g1, cu_s = O.qformer_window_pool(Hs[:1], [0, 1], Q, Wk, Wv, Wo, 4)
    assert cu_s.tolist() == [0, 3] and np.abs(g1 - (Wo @ (Wv @ Hs[0]))[None, :]).max() < 1e-12
    # one head, one query, two frames: p = sigmoid of the score difference
    q = rng.standard_normal((1, 32))
    s = (Wk @ Hs[:2].T).T @ q[0] / np.sqrt(32)
    p0 = 1 / (1 + np.exp(s[1] - s[0]))
    g2, _ = O.qformer_window_pool(Hs[:2], [0, 2], q, Wk, Wv, Wo, 1)
    want2 = Wo @ (p0 * (Wv @ Hs[0]) + (1 - p0) * (Wv @ Hs[1]))
    assert np.abs(g2[0] - want2).max() < 1e-12
    # a sharp query picks the frame with the largest score
    g3, _ = O.qformer_window_pool(Hs[:2], [0, 2], q * 1e4, Wk, Wv, Wo, 1)
    assert np.abs(g3[0] - Wo @ (Wv @ Hs[int(np.argmax(s))])).max() < 1e-9


def test_invariants():
    rng = np.random.default_rng(3)
    Q, Wk, Wv, Wo = _params(rng)
    Hs = rng.standard_normal((40, 24))
    cu = [0, 22, 40]
    g, cu_s = O.qformer_window_pool(Hs, cu, Q, Wk, Wv, Wo, 4)
    # frames inside a window may be permuted (attention is a set operation: there is no positional term)
    perm = Hs.copy()
    perm[0:15] = Hs[0:15][rng.permutation(15)]
    gp, _ = O.qformer_window_pool(perm, cu, Q, Wk, Wv, Wo, 4)
    assert np.abs(gp - g).max() < 1e-12
    # windows do not see each other, and never cross an utterance boundary
    other = Hs.copy()
    other[15:22] += 5.0                               # second (short) window of utterance 0
    go, _ = O.qformer_window_pool(other, cu, Q, Wk, Wv, Wo, 4)
    assert np.abs(go[:3] - g[:3]).max() == 0 and np.abs(go[6:] - g[6:]).max() == 0 and np.abs(go[3:6] - g[3:6]).max() > 1e-3
    # an utterance alone gives the rows it has in the batch
    ga, _ = O.qformer_window_pool(Hs[22:], [0, 18], Q, Wk, Wv, Wo, 4)
    assert np.array_equal(ga, g[cu_s[1]:])
    # rows: 3 per window, 5x fewer rows than frames for full windows
    assert cu_s.tolist() == [0, 6, 12] and g.shape[0] == 12
