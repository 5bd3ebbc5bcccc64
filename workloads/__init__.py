"""Seeded synthetic inputs shared by the oracle side and the HIP side.

This package only draws random inputs (CTC logits with a planted alignment,
random-init decoder weights, speech embeddings, prompt ids).  It contains none
of the method's arithmetic: no entropy, no collapse, no decoder math.
"""
from .configs import ModelCfg, Workload, WORKLOADS, get_workload  # noqa: F401
from .synth import (make_ctc_batch, make_model_weights, make_verify_inputs,  # noqa: F401
                    make_ctc_to_llm_map, CtcBatch, VerifyInputs)
