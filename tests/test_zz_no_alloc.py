"""ctc_gate_noalloc (the entry point for callers that cannot allocate) against ctc_gate, through the C ABI."""
import numpy as np
import pytest
import torch

from workloads import WORKLOADS, make_ctc_batch

pytestmark = pytest.mark.gpu


def _case(wl, ctx, n_utts):
    """Both entry points on the first n_utts utterances of the workload's batch; outputs must be identical."""
    from paper_2603_11243_amd.binding import ctc_gate_noalloc
    cb = make_ctc_batch(wl)
    cu = cb.cu_frames[:n_utts + 1]
    n = int(cu[-1])
    z = cb.logits[:n].cuda()
    ref = ctx.ctc_gate(z, cu, wl.blank_id, wl.tau_ctc)
    cu_dev = torch.from_numpy(np.ascontiguousarray(cu)).cuda()
    out = {"max_entropy": torch.full((n_utts,), -1.0, dtype=torch.float32, device="cuda"),
           "gate_pass": torch.full((n_utts,), 7, dtype=torch.uint8, device="cuda"),
           "draft_ctc": torch.full((n,), -1, dtype=torch.int32, device="cuda"),
           "draft_len": torch.full((n_utts,), -1, dtype=torch.int32, device="cuda")}
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    ctc_gate_noalloc(z, cu_dev, wl.blank_id, wl.tau_ctc, out)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    dl = ref["draft_len"].cpu().numpy()
    assert np.array_equal(out["draft_len"].cpu().numpy(), dl)
    assert np.array_equal(out["gate_pass"].cpu().numpy(), ref["gate_pass"].cpu().numpy())
    assert np.array_equal(out["max_entropy"].cpu().numpy(), ref["max_entropy"].cpu().numpy())     # same kernels: bitwise
    a, b = out["draft_ctc"].cpu().numpy(), ref["draft_ctc"].cpu().numpy()
    for u in range(n_utts):
        assert np.array_equal(a[cu[u]:cu[u] + dl[u]], b[cu[u]:cu[u] + dl[u]])
    return dl


def test_noalloc_gate_matches_ctc_gate_twice_second_call_smaller():
    from paper_2603_11243_amd.binding import Context, SsdError, ctc_gate_noalloc, NOALLOC_MAX_FRAMES
    wl = WORKLOADS["cfg3_1b_ragged64"]                 # bf16 scores, 64 ragged utterances, 40 % pass the gate
    ctx = Context()
    try:
        ctx.reserve(max_frames=1 << 16, max_utts=wl.B)
        dl = _case(wl, ctx, wl.B)
        assert dl.min() >= 0 and dl.max() > 0
        _case(wl, ctx, 5)                              # smaller input: stale scratch contents must not matter
        _case(WORKLOADS["cfg1_tiny_f32"], ctx, 4)      # fp32 scores
        # beyond the built-in scratch: refused with a clear message, nothing launched
        n = NOALLOC_MAX_FRAMES + 256
        z = torch.zeros((n, 8), dtype=torch.bfloat16, device="cuda")
        cu_dev = torch.tensor([0, n], dtype=torch.int32, device="cuda")
        out = {"max_entropy": torch.empty(1, device="cuda"), "gate_pass": torch.empty(1, dtype=torch.uint8, device="cuda"),
               "draft_ctc": torch.empty(n, dtype=torch.int32, device="cuda"), "draft_len": torch.empty(1, dtype=torch.int32, device="cuda")}
        with pytest.raises(SsdError, match="at most 262144"):
            ctc_gate_noalloc(z, cu_dev, 0, 0.7, out)
    finally:
        ctx.close()
