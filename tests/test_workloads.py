"""The synthetic generators: shapes, determinism, and that the oracle sees the intended structure."""
import numpy as np
import torch

from oracle import ssd_oracle as O
from workloads import WORKLOADS, make_ctc_batch, make_ctc_to_llm_map, make_model_weights, make_verify_inputs
from workloads.configs import scaled_down


def test_ctc_batch_shapes_and_determinism():
    wl = WORKLOADS["cfg3_1b_ragged64"]
    a, b = make_ctc_batch(wl), make_ctc_batch(wl)
    assert torch.equal(a.logits, b.logits) and np.array_equal(a.cu_frames, b.cu_frames)
    T = np.diff(a.cu_frames)
    assert a.logits.shape == (a.cu_frames[-1], 512) and a.logits.dtype == torch.bfloat16
    assert T.min() >= 50 and T.max() <= 500 and len(T) == 64
    assert a.confident.sum() == 26          # round(0.4 * 64)
    c = make_ctc_batch(wl, seed=7)
    assert not np.array_equal(a.cu_frames, c.cu_frames)


def test_oracle_gate_recovers_planted_structure():
    wl = WORKLOADS["cfg3_1b_ragged64"]
    cb = make_ctc_batch(wl)
    r = O.ctc_gate(cb.logits.float().numpy(), cb.cu_frames, wl.blank_id, wl.tau_ctc)
    assert np.array_equal(r["gate_pass"], cb.confident)
    for b in np.flatnonzero(cb.confident):
        assert np.array_equal(r["drafts"][b], cb.planted_tokens[b])
    lens = np.array([len(d) for d in r["drafts"]])
    planted = np.array([len(t) for t in cb.planted_tokens])
    assert (lens >= planted).all() and (lens <= planted * 1.3 + 2).all()


def test_tiny_workload_matches_config_text():
    wl = WORKLOADS["cfg1_tiny_f32"]
    cb = make_ctc_batch(wl)
    assert cb.logits.dtype == torch.float32 and cb.logits.shape == (480, 256)
    r = O.ctc_gate(cb.logits.numpy(), cb.cu_frames, 0, wl.tau_ctc)
    assert not r["gate_pass"].any()
    m = make_ctc_to_llm_map(wl)
    assert len(set(m.tolist())) == 256 and m.max() < 4096
    drafts = [m[d] for d in r["drafts"]]
    vi = make_verify_inputs(wl, cb.seconds, drafts)
    assert vi.speech_emb.shape == (120, 256) and list(np.diff(vi.cu_prompt)) == [10] * 4
    assert all(20 <= u <= 46 for u in np.diff(vi.cu_draft))
    w = make_model_weights(wl.model, wl.seed)
    assert w["layers"][1]["w_down"].shape == (256, 1024) and w["embed"].dtype == torch.float32
    assert abs(float(w["layers"][0]["wq"].std()) - 0.02) < 1e-3


def test_scaled_down_keeps_shapes():
    wl = scaled_down(WORKLOADS["cfg2_1b_b1"], n_layers=1)
    assert wl.model.d_model == 2048 and wl.model.n_layers == 1
