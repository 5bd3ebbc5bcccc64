"""GPU parity of the projector's windowed cross-attention (qformer_pool, through the C ABI) against the oracle."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import ssd_oracle as O
from workloads import WORKLOADS
from workloads.synth import make_ctc_head_batch, make_qformer_weights

pytestmark = pytest.mark.gpu


def _check(g_gpu, g_ref):
    """Rows are stored as bf16 (2^-9 relative rounding) from bf16 operands: elementwise within 2e-2 of the row's
    largest magnitude, and 1e-2 in relative L2 norm per row (a wrong window, head or query is O(1) in both)."""
    assert g_gpu.shape == g_ref.shape
    scale = np.abs(g_ref).max(axis=1, keepdims=True)
    assert (np.abs(g_gpu - g_ref) <= 2e-2 * scale).all(), float((np.abs(g_gpu - g_ref) / scale).max())
    rel = np.linalg.norm(g_gpu - g_ref, axis=1) / np.linalg.norm(g_ref, axis=1)
    assert rel.max() < 1e-2, float(rel.max())
    return float(rel.max())


@pytest.mark.parametrize("name,B,d_out", [("cfg3_1b_ragged64", 10, 2048), ("cfg5_3b_ragged128", 6, 3072), ("cfg1_tiny_f32", 2, 256)])
def test_qformer_pool_matches_oracle(name, B, d_out):
    """Paper shapes (1024-wide encoder states, 16 heads, windows of 15 frames, 3 queries) on ragged utterances
    whose lengths are mostly not multiples of 15; the third case has fewer than 128 frames in total (the few-row
    GEMM tiles)."""
    from paper_2603_11243_amd.binding import Context
    wl = replace(WORKLOADS[name], B=B, model=replace(WORKLOADS[name].model, dtype="bf16"))
    if name == "cfg1_tiny_f32":
        wl = replace(wl, seconds=(1.0, 2.5))
    hb = make_ctc_head_batch(wl, d_enc=1024, V_ctc=348)
    qw = make_qformer_weights(wl.seed, d_out=d_out)
    T = np.diff(hb.cu_frames)
    assert (T % 15 != 0).any()
    ctx = Context()
    try:
        ctx.set_qformer(*(qw[k].cuda() for k in ("q_proj", "w_k", "w_v", "w_o")), n_heads=16, window=15)
        ctx.reserve(max_frames=int(hb.cu_frames[-1]), max_utts=B)
        g, cu_s = ctx.qformer_pool(hb.enc_h.cuda(), hb.cu_frames)
        torch.cuda.synchronize()
        g2, _ = ctx.qformer_pool(hb.enc_h.cuda(), hb.cu_frames)            # same buffers, same answer
        torch.cuda.synchronize()
        assert torch.equal(g, g2)
    finally:
        ctx.close()
    ref, cu_ref = O.qformer_window_pool(hb.enc_h, hb.cu_frames, qw["q_proj"], qw["w_k"], qw["w_v"], qw["w_o"], 16, 15)
    assert np.array_equal(cu_s, cu_ref) and cu_s[-1] == 3 * sum(-(-int(t) // 15) for t in T)
    worst = _check(g.float().cpu().numpy(), ref)
    print(f"{wl.name}: {int(hb.cu_frames[-1])} frames -> {int(cu_s[-1])} rows, worst relative row error {worst:.2e}")


def test_qformer_pool_argument_errors():
    from paper_2603_11243_amd.binding import Context, SsdError
    ctx = Context()
    try:
        h = torch.zeros((30, 1024), dtype=torch.bfloat16, device="cuda")
        ctx._qformer = (3, 1024, 2048, 15)
        with pytest.raises(SsdError, match="no projector set"):
            ctx.qformer_pool(h, [0, 30])
        qw = make_qformer_weights(1)
        with pytest.raises(SsdError, match="pairs"):
            ctx.set_qformer(*(qw[k].cuda() for k in ("q_proj", "w_k", "w_v", "w_o")), n_heads=32)     # 3 x 32 score rows
        ctx.set_qformer(*(qw[k].cuda() for k in ("q_proj", "w_k", "w_v", "w_o")), n_heads=16)
        with pytest.raises(SsdError, match="workspace"):
            ctx.qformer_pool(h, [0, 30])
        ctx.reserve(max_frames=30, max_utts=2)
        with pytest.raises(SsdError, match="increase strictly"):
            ctx.qformer_pool(h, [0, 30, 30])
    finally:
        ctx.close()
