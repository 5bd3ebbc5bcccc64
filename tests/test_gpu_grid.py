"""GPU parity of the operating-point grids (Sec. 3.2) against the oracle."""
import numpy as np
import pytest
import torch

from oracle import ssd_oracle as O

pytestmark = pytest.mark.gpu


def test_gate_and_accept_grids_match_oracle():
    from paper_2603_11243_amd.binding import Context
    ctx = Context()
    ctx.reserve(max_frames=1024, max_utts=64)
    rng = np.random.default_rng(5)
    H = rng.uniform(0, 5, size=37).astype(np.float32)
    H[4] = np.float32(0.7); H[9] = np.float32(3.0)                        # equality fails
    U = rng.integers(0, 90, size=21); U[3] = 0
    cu = np.concatenate([[0], np.cumsum(U)]).astype(np.int32)
    lp = (-rng.exponential(1.3, size=int(cu[-1]))).astype(np.float32)
    lp[cu[5]] = np.float32(np.log(np.float64(np.float32(0.2))))          # equality fails
    tc = [0.7, 1.0, 2.0, 3.0]
    ts = [0.0, 0.1, 0.2, 0.5, 1.0]
    g = ctx.gate_grid(torch.from_numpy(H).cuda(), tc).cpu().numpy().astype(bool)
    a = ctx.accept_grid(torch.from_numpy(lp).cuda(), cu, ts)
    torch.cuda.synchronize()
    # the oracle decides on the same stored fp32 numbers; thresholds enter as the fp32 values the ABI takes
    lps = [lp[cu[b]:cu[b + 1]].astype(np.float64) for b in range(len(U))]
    ln_ts = [float(np.float32(np.log(np.float64(np.float32(t))))) if t > 0 else -np.inf for t in ts]
    want = O.threshold_grid(H.astype(np.float64), lps, [float(np.float32(t)) for t in tc],
                            [float(np.exp(x)) if np.isfinite(x) else 0.0 for x in ln_ts])
    assert np.array_equal(g, want["gate_pass"])
    got_len = a["accept_len"].cpu().numpy()
    # exp(log) round trips may move a threshold by an ulp: compare on the log scale directly
    for i, lt in enumerate(ln_ts):
        for b, x in enumerate(lps):
            bad = np.flatnonzero(~(x > lt))
            assert got_len[i, b] == (bad[0] if len(bad) else len(x))
    assert np.array_equal(a["all_accepted"].cpu().numpy().astype(bool), got_len == U[None, :])
    assert (got_len[:-1] >= got_len[1:]).all()
    assert np.array_equal(got_len[0], U) and (got_len[-1] == 0).all()
    ctx.close()


def test_measurement_aids_report_plausible_ceilings():
    """The two measured denominators of bench.py: an MFMA-only loop and a plain streaming read.  Both are
    bounded by the chip's nominal peaks (2.5 PFLOP/s, 8 TB/s) and must not come out absurdly low either;
    a buffer that is not 16-byte aligned is an argument error."""
    from paper_2603_11243_amd.binding import Context, SsdError
    ctx = Context()
    ctx.reserve(max_frames=200000, max_utts=64)         # the MFMA loop uses 513 KB of the workspace
    tf, ghz = ctx.measure_mfma_ceiling(2000)
    assert 300.0 < tf < 2500.0 and 0.5 < ghz < 2.6
    buf = torch.ones(1 << 28, dtype=torch.uint8, device="cuda")
    gbs = ctx.measure_hbm_read(buf, 3)
    assert 1000.0 < gbs < 16000.0                        # 256 MB may partly sit in the memory-side cache
    with pytest.raises(SsdError):
        ctx.measure_hbm_read(buf[1:], 1)
    ctx.close()
