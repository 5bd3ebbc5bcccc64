"""Comparison rules shared by the GPU parity tests.

Integer outputs (greedy path, drafts, lengths) are compared bit-exactly.  Decisions that
hinge on a floating-point comparison are compared exactly except where the oracle's margin
to the threshold is below the stated tolerance.
"""
import math

import numpy as np

TOL_H = 1e-4          # nats, frame entropy (fp32 from exactly widened inputs)
TOL_LOGP = {"bf16": 2e-2, "f32": 1e-4}


def check_gate_decisions(gate_pass_gpu, frame_entropy_oracle, cu_frames, tau, tol=TOL_H):
    for b in range(len(cu_frames) - 1):
        H = frame_entropy_oracle[cu_frames[b]:cu_frames[b + 1]]
        if gate_pass_gpu[b]:
            assert not (H >= tau + tol).any(), f"utt {b}: GPU passed the gate but a frame has H >= tau + tol"
        else:
            assert (H >= tau - tol).any(), f"utt {b}: GPU failed the gate but every frame has H < tau - tol"


def check_accept_len(accept_len_gpu, all_ok_gpu, logp_oracle, tau, tol):
    """logp_oracle: float64 array of one utterance."""
    ln_tau = math.log(tau) if tau > 0 else -math.inf
    U = len(logp_oracle)
    A = int(accept_len_gpu)
    assert 0 <= A <= U
    assert bool(all_ok_gpu) == (A == U)
    fails = logp_oracle <= ln_tau - tol
    passes = logp_oracle > ln_tau + tol
    assert not fails[:A].any(), "a clearly failing token lies inside the accepted prefix"
    assert A == U or not passes[A], "the token after the accepted prefix clearly passes"


def unambiguous(logp_oracle, tau, tol):
    ln_tau = math.log(tau)
    return not (np.abs(logp_oracle - ln_tau) <= tol).any()
