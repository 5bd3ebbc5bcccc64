"""GPU parity of ctc_head_gate (CTC output layer fused with the gate, through the C ABI) against the
oracle.  The scores are fp32 on the GPU and float64 in the oracle, so a frame whose two best scores
are closer than MARGIN has no unique greedy symbol at the kernel's precision: there the GPU's choice
must be one of the near-maximal symbols, and everything downstream of it (the collapse) is checked
for validity against the GPU's own path; everywhere else paths and drafts are compared exactly."""
import numpy as np
import pytest
import torch

from oracle import ssd_oracle as O
from tests.parity import TOL_H, check_gate_decisions
from workloads import WORKLOADS
from workloads.synth import make_ctc_head_batch

pytestmark = pytest.mark.gpu

MARGIN = 1e-4      # fp32 accumulation of <= 1024 exact bf16 products with |z| < 64: error well below 1e-5


@pytest.fixture(scope="module")
def ctx():
    from paper_2603_11243_amd.binding import Context
    c = Context()
    yield c
    c.close()


def _run_and_compare(ctx, enc_h, w, bias, cu, blank, tau):
    cu = np.asarray(cu, dtype=np.int32)
    B, n = len(cu) - 1, int(cu[-1])
    z = O.ctc_head_logits(enc_h, w, bias)
    ref = O.ctc_gate(z, cu, blank, tau)
    ctx.set_ctc_head(w.cuda(), None if bias is None else bias.cuda())
    ctx.reserve(max_frames=n, max_utts=B)
    out = ctx.ctc_head_gate(enc_h.cuda(), cu, blank, tau, want_frames=True)
    torch.cuda.synchronize()
    arg = out["frame_argmax"].cpu().numpy()
    H = out["frame_entropy"].cpu().numpy()
    top2 = np.partition(z, -2, axis=1)[:, -2:] if z.shape[1] > 1 else np.stack([np.full(n, -np.inf), z[:, 0]], 1)
    clear = (top2[:, 1] - top2[:, 0]) > MARGIN
    assert np.array_equal(arg[clear], ref["frame_argmax"][clear])
    assert (z[np.arange(n), arg] >= top2[:, 1] - MARGIN).all()          # near ties: any near-maximal symbol
    assert clear.mean() > 0.99
    assert np.abs(H - ref["frame_entropy"]).max() <= TOL_H
    dl = out["draft_len"].cpu().numpy()
    dc = out["draft_ctc"].cpu().numpy()
    for b in range(B):
        mine = O.collapse(arg[cu[b]:cu[b + 1]], blank)                   # valid collapse of the GPU's own path
        assert dl[b] == len(mine) and np.array_equal(dc[cu[b]:cu[b] + dl[b]], mine)
        if clear[cu[b]:cu[b + 1]].all():
            assert np.array_equal(mine, ref["drafts"][b])
    assert np.abs(out["max_entropy"].cpu().numpy() - ref["max_entropy"]).max() <= TOL_H
    gp = out["gate_pass"].cpu().numpy().astype(bool)
    check_gate_decisions(gp, ref["frame_entropy"], cu, tau)
    out2 = ctx.ctc_head_gate(enc_h.cuda(), cu, blank, tau, want_frames=False)   # internal per-frame scratch
    torch.cuda.synchronize()
    for k in ("draft_len", "gate_pass", "max_entropy"):
        assert torch.equal(out2[k], out[k])
    dc2 = out2["draft_ctc"].cpu().numpy()
    for b in range(B):
        assert np.array_equal(dc2[cu[b]:cu[b] + dl[b]], dc[cu[b]:cu[b] + dl[b]])
    return gp


@pytest.mark.parametrize("name,V", [("cfg2_1b_b1", 348), ("cfg3_1b_ragged64", 348), ("cfg3_1b_ragged64", 512),
                                    ("cfg4_1b_long_ml", 348)])
def test_head_gate_matches_oracle_on_workload_shapes(ctx, name, V):
    wl = WORKLOADS[name]
    hb = make_ctc_head_batch(wl, d_enc=1024, V_ctc=V)
    blank = min(wl.blank_id, V - 1)
    gp = _run_and_compare(ctx, hb.enc_h, hb.w_ctc, hb.bias, hb.cu_frames, blank, wl.tau_ctc)
    assert np.array_equal(gp, hb.confident)          # planted structure is far from the threshold


@pytest.mark.parametrize("V,d_enc,with_bias", [(8, 64, True), (40, 192, False), (64, 64, True), (65, 128, True),
                                               (256, 1024, True), (348, 1024, False), (520, 256, True),
                                               (1000, 320, True)])
def test_head_gate_symbol_counts_widths_and_ragged_tails(ctx, V, d_enc, with_bias):
    rng = np.random.default_rng(V * 7 + d_enc)
    T = [1, 3, 257, 300, 64, 700]
    cu = np.concatenate([[0], np.cumsum(T)])
    n = int(cu[-1])
    w = torch.from_numpy((rng.standard_normal((V, d_enc)) / np.sqrt(d_enc)).astype(np.float32)).bfloat16()
    bias = torch.from_numpy((0.3 * rng.standard_normal(V)).astype(np.float32)) if with_bias else None
    blank = V // 2
    lab = rng.integers(0, V, size=n)
    lab[rng.random(n) < 0.5] = blank
    lab = np.repeat(lab[::3], 3)[:n]                  # runs of repeated labels and blanks for the collapse
    wf = w.float().numpy()
    h = rng.standard_normal((n, d_enc)).astype(np.float32) * 2 + 12.0 * wf[lab] / (wf[lab] ** 2).sum(1, keepdims=True)
    _run_and_compare(ctx, torch.from_numpy(h).bfloat16(), w, bias, cu, blank, 0.7)


def test_head_gate_many_frames_takes_the_tall_tile(ctx):
    # more than 255 row tiles of 256 frames: the 256-row tile variant
    rng = np.random.default_rng(99)
    V, d_enc, B = 348, 128, 90
    T = rng.integers(600, 900, size=B)
    cu = np.concatenate([[0], np.cumsum(T)])
    n = int(cu[-1])
    assert n > 255 * 256
    w = torch.from_numpy((rng.standard_normal((V, d_enc)) / np.sqrt(d_enc)).astype(np.float32)).bfloat16()
    bias = torch.from_numpy((0.1 * rng.standard_normal(V)).astype(np.float32))
    wf = w.float().numpy()
    lab = np.repeat(rng.integers(0, V, size=n // 2 + 1), 2)[:n]
    boost = np.where(rng.random(n) < 0.5, 14.0, 6.0).astype(np.float32)
    h = rng.standard_normal((n, d_enc)).astype(np.float32) + boost[:, None] * wf[lab] / (wf[lab] ** 2).sum(1, keepdims=True)
    _run_and_compare(ctx, torch.from_numpy(h).bfloat16(), w, bias, cu, 0, 1.0)


def test_head_gate_uniform_and_one_hot_rows(ctx):
    # zero weight: every frame has softmax(bias); closed forms ln V (flat bias) and the one-peak entropy
    V, d_enc = 348, 64
    h = torch.randn(300, d_enc, generator=torch.Generator().manual_seed(1)).bfloat16()
    w = torch.zeros(V, d_enc, dtype=torch.bfloat16)
    ctx.set_ctc_head(w.cuda(), None)
    ctx.reserve(max_frames=300, max_utts=2)
    out = ctx.ctc_head_gate(h.cuda(), [0, 100, 300], 5, 6.0, want_frames=True)
    torch.cuda.synchronize()
    assert np.abs(out["frame_entropy"].cpu().numpy() - np.log(V)).max() <= TOL_H
    assert (out["frame_argmax"].cpu().numpy() == 0).all()            # lowest index among equal scores
    assert out["draft_len"].cpu().tolist() == [1, 1] and out["gate_pass"].cpu().tolist() == [1, 1]
    bias = torch.zeros(V)
    bias[200] = 30.0
    ctx.set_ctc_head(w.cuda(), bias.cuda())                            # replaces the first output layer
    out = ctx.ctc_head_gate(h.cuda(), [0, 100, 300], 200, 0.7, want_frames=True)
    torch.cuda.synchronize()
    assert out["frame_entropy"].cpu().abs().max().item() <= TOL_H
    assert (out["frame_argmax"].cpu().numpy() == 200).all()
    assert out["draft_len"].cpu().tolist() == [0, 0]                  # every frame is the blank


def test_head_gate_rejects_bad_calls():
    from paper_2603_11243_amd.binding import Context, SsdError
    c = Context()
    try:
        h = torch.zeros(4, 64, dtype=torch.bfloat16, device="cuda")
        c.reserve(max_frames=4, max_utts=1)
        with pytest.raises(SsdError):
            c.ctc_head_gate(h, [0, 4], 0, 1.0)                         # no output layer yet
        with pytest.raises(SsdError):
            c.set_ctc_head(torch.zeros(8, 48, dtype=torch.bfloat16, device="cuda"))    # d_enc not a multiple of 64
        c.set_ctc_head(torch.zeros(8, 64, dtype=torch.bfloat16, device="cuda"))
        with pytest.raises(SsdError):
            c.ctc_head_gate(h, [0, 4], 8, 1.0)                         # blank outside the symbols
        with pytest.raises(SsdError):
            c.ctc_head_gate(h, [0, 2, 2, 4], 0, 1.0)                   # an utterance without frames
        c.set_workspace(None)
        with pytest.raises(SsdError):
            c.ctc_head_gate(h, [0, 4], 0, 1.0)                         # no workspace
    finally:
        c.close()
