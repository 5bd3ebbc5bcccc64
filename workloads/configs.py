"""Shapes of the five synthetic workloads (stand-ins for the paper's corpora).

The paper evaluates on public speech corpora that are not available here; these
records only fix tensor shapes, length mixes and gate rates.  Rates: 25 CTC
frames per second of audio, 6 speech embeddings per second.
"""
from dataclasses import dataclass, replace
from typing import Tuple


@dataclass(frozen=True)
class ModelCfg:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    dtype: str = "bf16"          # "bf16" or "f32": storage type of weights and inputs

    @property
    def d_q(self):
        return self.n_q_heads * self.head_dim

    @property
    def d_kv(self):
        return self.n_kv_heads * self.head_dim

    def params_per_layer(self):
        d = self.d_model
        return d * self.d_q + 2 * d * self.d_kv + self.d_q * d + 3 * d * self.d_ff


@dataclass(frozen=True)
class Workload:
    name: str
    model: ModelCfg
    B: int                        # utterances
    V_ctc: int                    # CTC vocabulary including blank
    blank_id: int = 0
    seconds: Tuple[float, float] = (10.0, 10.0)   # uniform range of audio length
    frames_per_s: float = 25.0
    speech_per_s: float = 6.0
    speech_fixed: int = -1        # if >=0: S_b fixed, else round(speech_per_s * s)
    prompt_len: int = 16
    draft_tokens: Tuple[int, int] = (-1, -1)      # if >=0: uniform range of planted U_b
    draft_per_s: float = 4.0      # else planted U_b = round(draft_per_s * s)
    gate_rate: float = 0.0        # fraction of utterances planted confident
    corrupt_frac: float = 0.0     # fraction of draft positions replaced by random ids
    tau_ctc: float = 0.7
    seed: int = 0


TINY = ModelCfg(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64,
                d_ff=1024, vocab=4096, dtype="f32")
LLM_1B = ModelCfg(n_layers=24, d_model=2048, n_q_heads=16, n_kv_heads=8, head_dim=128,
                  d_ff=8192, vocab=49152)
LLM_1B_ML = replace(LLM_1B, vocab=100352)
LLM_3B = ModelCfg(n_layers=32, d_model=3072, n_q_heads=24, n_kv_heads=8, head_dim=128,
                  d_ff=8192, vocab=49152)

WORKLOADS = {
    "cfg1_tiny_f32": Workload("cfg1_tiny_f32", TINY, B=4, V_ctc=256, seconds=(4.8, 4.8),
                              speech_fixed=30, prompt_len=10, draft_tokens=(20, 40), seed=1000),
    "cfg2_1b_b1": Workload("cfg2_1b_b1", LLM_1B, B=1, V_ctc=512, seconds=(10.0, 10.0),
                           speech_fixed=60, prompt_len=16, draft_tokens=(30, 30), seed=2000),
    "cfg3_1b_ragged64": Workload("cfg3_1b_ragged64", LLM_1B, B=64, V_ctc=512, seconds=(2.0, 20.0),
                                 prompt_len=16, gate_rate=0.4, seed=3000),
    "cfg4_1b_long_ml": Workload("cfg4_1b_long_ml", LLM_1B_ML, B=16, V_ctc=2048, seconds=(30.0, 30.0),
                                speech_fixed=200, prompt_len=16, draft_tokens=(120, 120), seed=4000),
    "cfg5_3b_ragged128": Workload("cfg5_3b_ragged128", LLM_3B, B=128, V_ctc=512, seconds=(1.0, 30.0),
                                  prompt_len=16, gate_rate=0.3, corrupt_frac=0.1, seed=5000),
}


def get_workload(name: str) -> Workload:
    return WORKLOADS[name]


def scaled_down(wl: Workload, n_layers: int, B: int = None) -> Workload:
    """Same shapes with fewer layers / utterances (used by parity tests that need a
    CPU-affordable oracle run)."""
    m = replace(wl.model, n_layers=n_layers)
    return replace(wl, model=m, B=wl.B if B is None else B, name=f"{wl.name}_L{n_layers}")
