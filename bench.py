#!/usr/bin/env python3
"""Benchmark of the gate -> verify -> accept hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--only LEG] [--skip LEG,LEG]

A step is one pass of the whole path over one synthetic batch that is already resident in HBM:
ctc_gate -> (read gate flags and draft lengths; ssd_select_unconfident packs the inputs of the utterances
that failed the gate and maps CTC symbols to LLM ids) -> verify_forward -> accept_prefix.  Every kernel of a
step is the library's; torch only owns the buffers.  Prints ONE JSON line.

The default workload is the largest configuration (cfg5_3b_ragged128); the other four configurations are
timed as side entries of the same line (`other_configs`).  `--only LEG` runs one leg alone (for counter
runs under rocprofv3, which should contain nothing else); `--skip` leaves legs out.
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from workloads import (WORKLOADS, make_ctc_batch, make_ctc_to_llm_map, make_model_weights,  # noqa: E402
                       make_verify_inputs)

PEAK_MFMA_TFLOPS = 2500.0      # MI355X dense 16-bit matrix peak (bf16 and fp16)
PEAK_HBM_GBS = 8000.0
PEAK_F32_VALU_TFLOPS = 157.3   # the fp32 model runs on the vector ALUs

LEGS = ["main", "cpu_baseline", "mfma_ceiling", "hbm_ceiling", "ar_fallback", "gate_saturation", "ctc_head", "qformer",
        "other_configs", "two_phase", "library_gemm"]

# HBM-side traffic of the dominant kernel (gate/up projection) per launch, from two rocprofv3 --pmc runs of
# `bench.py --only main --workload NAME` (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch, averaged over the launches
# of the kernel on M rows), each scaled by what the same counter reads for a plain 1 GiB device copy
# (`--copy-reference`).  Every entry names the committed summary it was read from.
MEASURED_TRAFFIC = {
    "cfg5_3b_ragged128": {"bytes": (1082288.8 * 2.0 + 238764.1 * 1.0) * 1024.0,    # average launch (full layers and the last layer's)
                          "source": "profiles/pmc_traffic_bench_cfg5_3b_ragged128.md"},
    "cfg3_1b_ragged64": {"bytes": (338432.4 * 2.0 + 82304.0 * 1.0) * 1024.0,       # a full layer (5144 rows)
                         "source": "profiles/pmc_traffic_gemm_gate_up_cfg3.md"},
    # ctc_gate at saturation size, both kernels of a call (scores read once; entropies and labels written, then read back)
    "gate_saturation_V512_bfloat16": {"bytes": ((781270.2 + 6478.5) * 2.0 + 12228.8 + 400.6) * 1024.0,
                                      "source": "profiles/ctc_gate_saturation_stats_and_traffic.md"},
}


def tau_for(wl, q=1.9):
    s = 0.02 * np.sqrt(wl.model.d_model)
    return float(np.exp(-np.log(wl.model.vocab) - s * s / 2 - q * s))


class Step:
    """Everything one step needs, prepared once; `run()` enqueues one step and returns its outputs."""

    def __init__(self, wl, ctx, device):
        self.wl, self.ctx, self.device = wl, ctx, device
        self.cb = make_ctc_batch(wl)
        self.logits = self.cb.logits.to(device)
        self.table = torch.from_numpy(make_ctc_to_llm_map(wl)).to(device)
        self.cu_frames = self.cb.cu_frames
        B, n_frames = wl.B, int(self.cu_frames[-1])
        # Inputs of the verify pass exist for every utterance; a step uses those of the utterances
        # that fail the gate.  Speech rows: round(6 * seconds) (or the fixed count), prompt ids random.
        self.vi_all = make_verify_inputs(wl, self.cb.seconds, [np.zeros(0, np.int32)] * B, device=device)
        self.prompt_ids = torch.from_numpy(self.vi_all.prompt_ids).to(device)
        nS, nP = int(self.vi_all.cu_speech[-1]), int(self.vi_all.cu_prompt[-1])
        max_tok = nS + nP + n_frames                                   # a draft is at most T tokens
        ctx.reserve(max_frames=n_frames, max_tokens=max_tok, max_verify_rows=n_frames, max_utts=B)
        m = wl.model
        # every buffer a step writes, allocated once at its largest size
        self.gate_out = None
        self.sel_buf = {"speech": torch.empty((nS, m.d_model), dtype=self.vi_all.speech_emb.dtype, device=device),
                        "prompt": torch.empty(nP, dtype=torch.int32, device=device),
                        "draft_ids": torch.empty(n_frames, dtype=torch.int32, device=device)}
        self.hv_buf = torch.empty((n_frames, m.d_model), dtype=ctx.act_dtype, device=device)
        self.acc_buf = {"draft_logp": torch.empty(n_frames, dtype=torch.float32, device=device),
                        "accept_len": torch.empty(B, dtype=torch.int32, device=device),
                        "all_accepted": torch.empty(B, dtype=torch.uint8, device=device)}

    def run(self, tau_slm):
        wl, ctx, vi = self.wl, self.ctx, self.vi_all
        g = ctx.ctc_gate(self.logits, self.cu_frames, wl.blank_id, wl.tau_ctc, out=self.gate_out)
        self.gate_out = g
        # the caller has to know which utterances go on and how long their drafts are: two small D2H copies
        gate_pass = g["gate_pass"].cpu().numpy()
        draft_len = g["draft_len"].cpu().numpy()
        fail = np.flatnonzero(gate_pass == 0)
        if len(fail) == 0:
            return g, None, None, 0
        sel = ctx.select_unconfident(fail, self.cu_frames, draft_len, g["draft_ctc"], self.table, vi.speech_emb,
                                     vi.cu_speech, self.prompt_ids, vi.cu_prompt, out=self.sel_buf)
        Mv, Bv = int(sel["cu_draft"][-1]), len(fail)
        hv = ctx.verify_forward(sel["speech"], sel["cu_speech"], sel["prompt"], sel["cu_prompt"], sel["draft_ids"],
                                sel["cu_draft"], out=self.hv_buf[:Mv])
        acc = ctx.accept_prefix(hv, sel["draft_ids"], sel["cu_draft"], tau_slm,
                                out={"draft_logp": self.acc_buf["draft_logp"][:Mv], "accept_len": self.acc_buf["accept_len"][:Bv],
                                     "all_accepted": self.acc_buf["all_accepted"][:Bv]})
        meta = {"fail": fail, "cu_s": sel["cu_speech"], "cu_p": sel["cu_prompt"], "cu_d": sel["cu_draft"],
                "speech": sel["speech"], "prompt": sel["prompt"], "draft_ids": sel["draft_ids"]}
        return g, acc, meta, Mv


def step_flops(m, meta):
    """Algorithmic flops of one verify_forward + accept_prefix: projections (all rows, except that after the attention
    of the last layer only the verification rows continue), the causal half of attention, the LM head on the draft
    positions only."""
    S, P, U = np.diff(meta["cu_s"]), np.diff(meta["cu_p"]), np.diff(meta["cu_d"])
    n = (S + P + U).astype(np.float64)
    M, Mv, L = float(n.sum()), float(U.sum()), m.n_layers
    qkv = m.d_model * (m.d_q + 2 * m.d_kv)
    rest = m.params_per_layer() - qkv
    proj = 2.0 * (L * M * qkv + ((L - 1) * M + Mv) * rest)
    attn = float(L * (4.0 * (n * (n + 1) / 2) * m.head_dim * m.n_q_heads).sum())
    head = 2.0 * Mv * m.vocab * m.d_model
    return {"projections": proj, "attention": attn, "lm_head": head, "total": proj + attn + head, "M": int(M), "Mv": int(Mv)}


def weight_bytes(m):
    return (2.0 if m.dtype == "bf16" else 4.0) * (m.n_layers * m.params_per_layer() + m.vocab * m.d_model)


def run_workload(wl, ctx, device, steps, warmup, detail=True):
    """Times `steps` steps of the whole path on one workload; returns the metrics and the live state."""
    m = wl.model
    step = Step(wl, ctx, device)
    tau = tau_for(wl)
    for _ in range(max(warmup, 1)):
        g, acc, meta, n_draft = step.run(tau)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        g, acc, meta, n_draft = step.run(tau)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    fl = step_flops(m, meta)
    out = {"ms_per_step": dt * 1e3, "verified_draft_tokens_per_s": n_draft / dt, "utterances_per_s": wl.B / dt,
           "decoder_rows": fl["M"], "draft_tokens": n_draft, "verified_utterances": len(meta["fail"]),
           "ctc_frames": int(step.cu_frames[-1])}
    # verify_forward + accept_prefix alone, timed with HIP events through the library on its own stream
    # (one span per call: the event pair brackets the whole forward, not single kernels)
    t1 = time.perf_counter()
    for _ in range(steps):
        hv = ctx.verify_forward(meta["speech"], meta["cu_s"], meta["prompt"], meta["cu_p"], meta["draft_ids"], meta["cu_d"],
                                out=step.hv_buf[:fl["Mv"]])
        ctx.accept_prefix(hv, meta["draft_ids"], meta["cu_d"], tau)
    torch.cuda.synchronize()
    dt_va = (time.perf_counter() - t1) / steps
    out["verify_accept_ms"] = dt_va * 1e3
    out["verify_accept_tokens_per_s"] = n_draft / dt_va
    if m.dtype == "bf16" and fl["M"] > 310:
        tf = fl["total"] / dt_va / 1e12
        out["verify_roofline"] = {"bound": "mfma", "what": "verify_forward + accept_prefix, all algorithmic flops over the time of the two calls",
                                  "achieved": tf, "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": tf / PEAK_MFMA_TFLOPS,
                                  "flops": fl}
    elif m.dtype == "bf16":
        gbs = weight_bytes(m) / dt_va / 1e9
        out["verify_roofline"] = {"bound": "hbm", "what": "verify_forward + accept_prefix: every weight streamed once per step",
                                  "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                                  "algorithmic_bytes_per_step": weight_bytes(m)}
    else:
        tf = fl["total"] / dt_va / 1e12
        out["verify_roofline"] = {"bound": "alu", "what": "fp32 model on the vector ALUs (no fp32 matrix path is used); "
                                  "at 285 rows the step is launch latency, not arithmetic",
                                  "achieved": tf, "peak": PEAK_F32_VALU_TFLOPS, "unit": "TFLOP/s", "frac": tf / PEAK_F32_VALU_TFLOPS}
    if detail:
        acc_len = acc["accept_len"].cpu().numpy()
        out["gate_pass_rate"] = float(g["gate_pass"].float().mean().cpu())
        out["full_accept_rate"] = float(acc["all_accepted"].float().mean().cpu())
        out["mean_accepted_prefix_frac"] = float(np.mean(acc_len / np.maximum(np.diff(meta["cu_d"]), 1)))
    return out, step, meta, tau, fl


def dominant_kernel(ctx, step, tau, meta, fl, m, steps):
    """HIP-event time of the dominant kernel (gate/up projection) and of every kernel class, in untimed extra steps
    of the same work (the timed region itself records no events)."""
    ctx.profile_select("gemm_gate_up")
    for _ in range(steps):
        step.run(tau)
    dom_ms, dom_n = ctx.profile_read()["gemm_gate_up"]
    ctx.profile_select(-1)
    step.run(tau)
    breakdown = {k: round(v[0], 4) for k, v in ctx.profile_read().items()}
    ctx.profile_select(-2)
    M, Mv, L = fl["M"], fl["Mv"], m.n_layers
    rows_avg = ((L - 1) * M + Mv) / L
    flops = 2.0 * rows_avg * m.d_model * 2 * m.d_ff
    avg_ms = dom_ms / max(dom_n, 1)
    tf = flops / (avg_ms * 1e-3) / 1e12 if dom_n else 0.0
    qkv_params = m.d_model * (m.d_q + 2 * m.d_kv)
    per = {"gemm_qkv": 2.0 * L * M * qkv_params, "gemm_o": 2.0 * L * rows_avg * m.d_model * m.d_q,
           "gemm_gate_up": 2.0 * L * rows_avg * m.d_model * 2 * m.d_ff, "gemm_down": 2.0 * L * rows_avg * m.d_model * m.d_ff}
    gemm_ms = sum(breakdown[k] for k in per)
    res = {"roofline": {"bound": "mfma", "kernel": "gemm_mfma16_kernel<EpiSwiglu> (gate/up projection + SiLU*mul)",
                        "achieved": tf, "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": tf / PEAK_MFMA_TFLOPS,
                        "traffic": None, "traffic_source": None,
                        "traffic_unit": "bytes per launch (L2<->fabric, incl. Infinity Cache hits)",
                        "algorithmic_bytes": 2.0 * (rows_avg * m.d_model + 2 * m.d_ff * m.d_model + rows_avg * m.d_ff),
                        "rows_per_launch": {"layers_before_last": M, "last_layer": Mv, "average": rows_avg},
                        "avg_launch_ms": avg_ms, "launches_timed": dom_n, "flops_per_launch": flops,
                        "timed_in": f"{steps} extra steps after the timed region (HIP events on the library's stream)"},
           "breakdown_ms_per_step": breakdown,
           "all_projection_gemms": {"tflops": sum(per.values()) / (gemm_ms * 1e-3) / 1e12 if gemm_ms else None,
                                    "frac_of_peak": sum(per.values()) / (gemm_ms * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS if gemm_ms else None},
           "projection_tflops": {k: (f / (breakdown[k] * 1e-3) / 1e12 if breakdown.get(k) else None) for k, f in per.items()}}
    if breakdown.get("lmhead_accept"):
        t_acc = breakdown["lmhead_accept"] * 1e-3
        acc_flops = 2.0 * Mv * m.vocab * m.d_model
        acc_bytes = 2.0 * (m.vocab * m.d_model + Mv * m.d_model) + 4.0 * Mv
        if Mv > 310:
            res["accept_roofline"] = {"bound": "mfma", "achieved": acc_flops / t_acc / 1e12, "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                                      "frac": acc_flops / t_acc / 1e12 / PEAK_MFMA_TFLOPS, "rows": Mv, "ms": breakdown["lmhead_accept"],
                                      "logit_bytes_never_written": 4.0 * Mv * m.vocab}
        else:
            res["accept_roofline"] = {"bound": "hbm", "achieved": acc_bytes / t_acc / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                      "frac": acc_bytes / t_acc / 1e9 / PEAK_HBM_GBS, "rows": Mv, "ms": breakdown["lmhead_accept"],
                                      "logit_bytes_never_written": 4.0 * Mv * m.vocab}
    return res


def cpu_baseline(wl, step, weights, meta, budget_rows):
    """The oracle, as it stands, on this machine's host cores, over a bounded sample of the same batch (median-length
    utterances up to budget_rows decoder rows).  The oracle widens each layer's weights itself."""
    from oracle import ssd_oracle as O
    import threadpoolctl
    cores = max((p["num_threads"] for p in threadpoolctl.threadpool_info() if p.get("user_api") == "blas"), default=1)
    fail = meta["fail"]
    lens = np.diff(meta["cu_s"]) + np.diff(meta["cu_p"]) + np.diff(meta["cu_d"])
    order = np.argsort(-lens)
    pick, tok = [], 0
    for k in order[len(order) // 2:]:                       # start from median-length utterances
        if tok + lens[k] > budget_rows and pick:
            break
        pick.append(int(k)); tok += int(lens[k])
    cu = lambda a: np.concatenate([[0], np.cumsum(a)]).astype(np.int32)
    sp = torch.cat([meta["speech"][meta["cu_s"][k]:meta["cu_s"][k + 1]] for k in pick]).cpu()
    pr = np.concatenate([meta["prompt"][meta["cu_p"][k]:meta["cu_p"][k + 1]].cpu().numpy() for k in pick])
    dr = np.concatenate([meta["draft_ids"][meta["cu_d"][k]:meta["cu_d"][k + 1]].cpu().numpy() for k in pick])
    cs, cp, cd = (cu(np.diff(meta[n])[pick]) for n in ("cu_s", "cu_p", "cu_d"))
    utt = fail[pick]
    rows = np.concatenate([np.arange(step.cu_frames[b], step.cu_frames[b + 1]) for b in utt])
    z = step.cb.logits[rows].float().numpy()
    cuf = cu([step.cu_frames[b + 1] - step.cu_frames[b] for b in utt])
    t0 = time.perf_counter()
    O.ctc_gate(z, cuf, wl.blank_id, wl.tau_ctc)
    lp = O.draft_logp(weights, wl.model, sp, cs, pr, cp, dr, cd)
    for x in lp:
        O.accept_prefix(x, tau_for(wl))
    dt = time.perf_counter() - t0
    n_draft = int(cd[-1])
    return {"value": n_draft / dt, "unit": "verified draft tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{len(pick)} of {len(fail)} verified utterances of {wl.name} ({n_draft} draft tokens, {tok} decoder rows), "
                      f"gate+verify+accept in float64 numpy, {dt:.1f} s",
            "utterances_per_s": len(pick) / dt}


def gate_saturation_leg(ctx, wl, device):
    """Bandwidth of ctc_gate on a working set far larger than the 256 MB Infinity Cache: the workload's
    frame shape (V_ctc, storage type) repeated to about 1.6 GB, 400-frame utterances, HIP events."""
    V = wl.V_ctc
    dt = torch.bfloat16 if wl.model.dtype == "bf16" else torch.float32
    T = 400
    n_utts = max(1, int(1.6e9 / (V * (2 if dt == torch.bfloat16 else 4))) // T)
    n_rows = n_utts * T
    cu = np.arange(n_utts + 1, dtype=np.int32) * T
    z = torch.randn(n_rows, V, device=device, dtype=torch.float32).to(dt)
    z[:, 7] += 6.0
    ctx.reserve(max_frames=n_rows, max_utts=n_utts)
    out = ctx.ctc_gate(z, cu, wl.blank_id, wl.tau_ctc)
    torch.cuda.synchronize()
    ctx.profile_select("gate")
    for _ in range(10):
        ctx.ctc_gate(z, cu, wl.blank_id, wl.tau_ctc, out=out)
    ms, n = ctx.profile_read()["gate"]
    ctx.profile_select(-2)
    nbytes = z.numel() * z.element_size() + n_rows * 12          # scores in; entropy, argmax, draft slot out
    gbs = nbytes / (ms / n * 1e-3) / 1e9
    tr = MEASURED_TRAFFIC.get("gate_saturation_V%d_%s" % (V, str(dt).replace("torch.", "")))
    return {"bound": "hbm", "kernel": "ctc_gate (frames kernel + per-utterance kernel)", "achieved": gbs,
            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS, "avg_call_ms": ms / n,
            "frames": n_rows, "V_ctc": V, "storage": str(dt).replace("torch.", ""), "bytes_per_frame": V * z.element_size() + 12,
            "algorithmic_bytes": nbytes, "traffic": tr["bytes"] if tr else None, "traffic_source": tr["source"] if tr else None}


def ctc_head_leg(ctx, wl, device, d_enc=1024, V=348):
    """Output layer of the CTC encoder fused with the gate (1024-wide states, 348 symbols), next to
    the same work done unfused: a library GEMM that stores bf16 scores, then ctc_gate on them.
    About 0.8 GB of encoder states (400-frame utterances), HIP events through the library's profiler."""
    if wl.model.dtype != "bf16":
        return None
    T = 400
    n_utts = int(0.8e9 / (d_enc * 2)) // T
    n_rows = n_utts * T
    cu = np.arange(n_utts + 1, dtype=np.int32) * T
    gen = torch.Generator(device=device)
    gen.manual_seed(5)
    w = (torch.randn(V, d_enc, device=device, generator=gen) / d_enc ** 0.5).bfloat16()
    bias = 0.1 * torch.randn(V, device=device, generator=gen)
    lab = torch.randint(0, V, (n_rows,), device=device, generator=gen)
    h = torch.randn(n_rows, d_enc, device=device, generator=gen)
    h += 8.0 * w.float()[lab] / (w.float()[lab] ** 2).sum(1, keepdim=True)
    h = h.bfloat16()
    del lab
    blank = min(wl.blank_id, V - 1)
    ctx.set_ctc_head(w, bias)
    ctx.reserve(max_frames=n_rows, max_utts=n_utts)
    ctx.ctc_head_gate(h, cu, blank, wl.tau_ctc)
    torch.cuda.synchronize()
    ctx.profile_select("ctc_head_gate")
    for _ in range(10):
        ctx.ctc_head_gate(h, cu, blank, wl.tau_ctc)
    ms, n = ctx.profile_read()["ctc_head_gate"]
    ctx.profile_select(-2)
    fused_ms = ms / n
    # unfused: scores through memory (library GEMM, padded to a 16-byte row for the gate kernel)
    Vs = (V + 7) // 8 * 8
    wp = torch.zeros(Vs, d_enc, device=device, dtype=torch.bfloat16)
    wp[:V] = w
    bp = torch.full((Vs,), -1e30, device=device)
    bp[:V] = bias
    z = torch.empty(n_rows, Vs, device=device, dtype=torch.bfloat16)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    def unfused():
        torch.addmm(bp.bfloat16(), h, wp.t(), out=z)
        return ctx.ctc_gate(z, cu, blank, wl.tau_ctc)
    unfused()
    torch.cuda.synchronize()
    ev[0].record()
    for _ in range(10):
        unfused()
    ev[1].record()
    torch.cuda.synchronize()
    unfused_ms = ev[0].elapsed_time(ev[1]) / 10
    flops = 2.0 * n_rows * d_enc * V
    tf = flops / (fused_ms * 1e-3) / 1e12
    return {"frames": n_rows, "d_enc": d_enc, "V_ctc": V, "ms_per_call": fused_ms, "frames_per_s": n_rows / (fused_ms * 1e-3),
            "unfused_library_gemm_plus_gate_ms": unfused_ms, "speedup_vs_unfused": unfused_ms / fused_ms,
            "roofline": {"bound": "mfma", "kernel": "ctc_head_partials_kernel (+ merge and per-utterance kernels)",
                         "achieved": tf, "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": tf / PEAK_MFMA_TFLOPS,
                         "flops_per_call": flops, "note": "348 symbols occupy 384 MFMA rows: 91 % of the issued flops are algorithmic"},
            "bytes_per_frame": {"fused": d_enc * 2 + 16 * ((V + 63) // 64) * 2 + 12, "unfused": d_enc * 2 + 2 * Vs * 2 + 12}}


def qformer_leg(ctx, wl, device, d_enc=1024, d_h=1024, n_heads=16, window=15, n_q=3):
    """The projector's windowed cross-attention (15 frames -> 3 queries) as the producer of the acoustic embeddings:
    about 0.8 GB of encoder states in 400-frame utterances, HIP events through the library's profiler."""
    if wl.model.dtype != "bf16":
        return None
    from workloads.synth import make_qformer_weights
    T = 400
    n_utts = int(0.8e9 / (d_enc * 2)) // T
    n_rows = n_utts * T
    cu = np.arange(n_utts + 1, dtype=np.int32) * T
    gen = torch.Generator(device=device)
    gen.manual_seed(6)
    h = torch.randn(n_rows, d_enc, device=device, generator=gen).bfloat16()
    qw = make_qformer_weights(wl.seed, n_q=n_q, d_h=d_h, d_enc=d_enc, d_out=wl.model.d_model, device=device)
    ctx.set_qformer(qw["q_proj"], qw["w_k"], qw["w_v"], qw["w_o"], n_heads=n_heads, window=window)
    ctx.reserve(max_frames=n_rows, max_utts=n_utts)
    g, cu_s = ctx.qformer_pool(h, cu)
    torch.cuda.synchronize()
    ctx.profile_select("qformer_pool")
    for _ in range(10):
        ctx.qformer_pool(h, cu, out=g)
    ms, n = ctx.profile_read()["qformer_pool"]
    ctx.profile_select(-2)
    ms /= n
    S = int(cu_s[-1])
    flops = 2.0 * n_rows * d_enc * (n_q * n_heads + d_h) + 2.0 * S * d_h * wl.model.d_model
    tf = flops / (ms * 1e-3) / 1e12
    return {"frames": n_rows, "speech_rows": S, "d_enc": d_enc, "d_h": d_h, "d_out": wl.model.d_model, "ms_per_call": ms,
            "frames_per_s": n_rows / (ms * 1e-3),
            "roofline": {"bound": "mfma", "kernel": "two gemm_mfma16 launches (scores | values, output projection) + qformer_pool_kernel",
                         "achieved": tf, "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": tf / PEAK_MFMA_TFLOPS, "flops_per_call": flops}}


def ar_fallback_leg(ctx, wl, meta, tau, n_steps=16):
    """Eq. 6 after the timed path: verify with the K/V cache, accept with greedy tokens, then n_steps of
    greedy continuation for the utterances whose draft was not fully accepted.  A decode step streams
    every layer's weights and the LM head once, so it is graded against HBM bandwidth."""
    m = wl.model
    S, P, U = np.diff(meta["cu_s"]), np.diff(meta["cu_p"]), np.diff(meta["cu_d"])
    cap = S + P + U + n_steps + 1
    kv_start = np.concatenate([[0], np.cumsum(cap)[:-1]]).astype(np.int32)
    ctx.set_kv_cache(int(cap.sum()))
    ctx.reserve(ar_utts=len(U), ar_steps=n_steps)
    hv = ctx.verify_forward(meta["speech"], meta["cu_s"], meta["prompt"], meta["cu_p"], meta["draft_ids"], meta["cu_d"],
                            kv_start=kv_start)
    acc = ctx.accept_prefix(hv, meta["draft_ids"], meta["cu_d"], tau, want_greedy=True)
    acc_len = acc["accept_len"].cpu().numpy()
    rej = np.flatnonzero(acc_len < U)
    if len(rej) == 0:
        return None
    idx = torch.from_numpy((meta["cu_d"][:-1][rej] + acc_len[rej]).astype(np.int64)).to(hv.device)
    first = acc["greedy_tok"][idx].contiguous()
    ctx_len = (S + P + acc_len)[rej].astype(np.int32)
    out = ctx.ar_fallback(kv_start[rej], ctx_len, first, n_steps)           # warm-up
    torch.cuda.synchronize()
    ctx.profile_select("ar_fallback")
    for _ in range(3):
        ctx.ar_fallback(kv_start[rej], ctx_len, first, n_steps, out=out)
    ms, n = ctx.profile_read()["ar_fallback"]
    ctx.profile_select(-2)
    step_ms = ms / n / n_steps
    gbs = weight_bytes(m) / (step_ms * 1e-3) / 1e9
    return {"rejected_utterances": int(len(rej)), "steps": n_steps, "ms_per_step": step_ms,
            "tokens_per_s": len(rej) / (step_ms * 1e-3),
            "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                         "algorithmic_bytes_per_step": weight_bytes(m)}}


def library_gemm_leg(m, M, device, iters=30):
    """The four projection shapes of one layer as plain library GEMMs (torch.matmul = hipBLASLt, IEEE half, no
    epilogue: no RoPE, SiLU*mul or residual add), next to which the fused kernels of this library are read.
    Operands are distributed like the real ones: normalised activations, N(0, 0.02^2) weights scaled by 2^9."""
    shapes = {"gemm_qkv": (m.d_q + 2 * m.d_kv, m.d_model), "gemm_o": (m.d_model, m.d_q),
              "gemm_gate_up": (2 * m.d_ff, m.d_model), "gemm_down": (m.d_model, m.d_ff)}
    gen = torch.Generator(device=device)
    gen.manual_seed(11)
    out = {}
    for name, (N, K) in shapes.items():
        a = torch.randn(M, K, device=device, generator=gen).half()
        w = (torch.randn(N, K, device=device, generator=gen) * (0.02 * 512)).half()
        for _ in range(3):
            c = a @ w.t()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        torch.cuda.synchronize()
        ev[0].record()
        for _ in range(iters):
            c = a @ w.t()
        ev[1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[1]) / iters
        out[name] = {"us": ms * 1e3, "tflops": 2.0 * M * N * K / (ms * 1e-3) / 1e12}
        del a, w, c
    return out


def other_configs_leg(main_name, device, steps):
    """The configurations that are not the headline, each on its own model (cfg2 runs on the model cfg3 was built
    with: same decoder shape, and time does not depend on the values).  MFMA roofline for the batched bf16
    configurations, HBM (weight streaming) for the single-utterance one, vector ALU for the fp32 one."""
    from paper_2603_11243_amd.binding import Context
    out = {}
    shared = None
    for name in ("cfg3_1b_ragged64", "cfg2_1b_b1", "cfg4_1b_long_ml", "cfg1_tiny_f32"):
        if name == main_name:
            continue
        wl = WORKLOADS[name]
        if name == "cfg2_1b_b1" and shared is not None:
            ctx = shared
        else:
            if shared is not None:
                shared.close()
                shared = None
            ctx = Context(wl.model, make_model_weights(wl.model, wl.seed, device=device), device=device)
        n = steps if wl.model.dtype == "bf16" and wl.B > 1 else 5 * steps
        res, step, meta, tau, fl = run_workload(wl, ctx, device, n, 3, detail=False)
        if wl.model.dtype == "bf16" and fl["M"] > 310:
            dom = dominant_kernel(ctx, step, tau, meta, fl, wl.model, max(2, n // 4))
            res["roofline"] = dom["roofline"]
            res["all_projection_gemms"] = dom["all_projection_gemms"]
        out[name] = res
        del step
        if name == "cfg3_1b_ragged64":
            shared = ctx
        else:
            if ctx is not shared:
                ctx.close()
    if shared is not None:
        shared.close()
    return out


def two_phase_leg(ctx, wl, step, tau, device, budgets=(5000, 20000, 50000), n_steps=8):
    """Sec. 3.2: length-sorted bins under a token budget, verification and fallback batched separately.  Reports
    utterances per second against the budget for the two ways of carrying an utterance from one phase to the
    other (see paper_2603_11243_amd/pipeline.py): the paper's (acoustic embeddings parked in pinned host memory,
    fallback bins re-run the prompt) and the resident one (K/V cache kept in HBM)."""
    from paper_2603_11243_amd.pipeline import TwoPhaseDecoder
    out = {"n_fallback_steps": n_steps, "budgets": {}}
    for budget in budgets:
        row = {}
        for mode in ("offload", "resident"):
            dec = TwoPhaseDecoder(ctx, wl, step.logits, step.cu_frames, step.table, step.vi_all.speech_emb, step.vi_all.cu_speech,
                                  step.prompt_ids, step.vi_all.cu_prompt, budget=budget, mode=mode, n_steps=n_steps)
            dec.run(tau)                                   # warm-up (buffers, staging)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            reps = 3
            for _ in range(reps):
                r = dec.run(tau)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / reps
            row[mode] = {"ms": dt * 1e3, "utterances_per_s": wl.B / dt, "verify_bins": r["verify_bins"],
                         "fallback_bins": r["fallback_bins"], "rejected": r["rejected"],
                         "offloaded_MB": r["offloaded_bytes"] / 1e6}
        out["budgets"][str(budget)] = row
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg5_3b_ragged128", choices=list(WORKLOADS))
    ap.add_argument("--only", default=None, choices=LEGS, help="run this leg alone (with the set-up it needs)")
    ap.add_argument("--skip", default="", help="comma-separated legs to leave out")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--main-only", action="store_true", help="same as --only main")
    ap.add_argument("--cpu-budget-rows", type=int, default=900)
    ap.add_argument("--copy-reference", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy five times (scale reference for --pmc counters)")
    ap.add_argument("--mfma-ceiling-only", action="store_true",
                    help="only run the MFMA-only ceiling kernel (a kernel whose matrix cores never idle: the 100 % mark "
                         "for the MFMA-busy counters of a --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on ONE GPU (utterance-sharded data parallelism needs no collectives and is "
              "not built); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    from paper_2603_11243_amd.binding import Context
    device = torch.device("cuda:0")
    if args.mfma_ceiling_only:
        wl = WORKLOADS["cfg1_tiny_f32"]
        ctx = Context(wl.model, make_model_weights(wl.model, wl.seed, device=device), device=device)
        ctx.reserve(max_frames=4096, max_tokens=4096, max_verify_rows=1024, max_utts=8)     # the kernel's 0.5 MB of workspace
        print(json.dumps(ctx.measure_mfma_ceiling()))
        return
    if args.copy_reference:
        a = torch.full((1 << 30,), 3, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        return
    skip = set(x for x in args.skip.split(",") if x)
    if args.no_cpu_baseline:
        skip.add("cpu_baseline")
    only = "main" if args.main_only else args.only
    want = lambda leg: (only == leg) if only else (leg not in skip)

    wl = WORKLOADS[args.workload]
    m = wl.model
    if only == "gate_saturation":                      # needs no model
        ctx = Context(device=device)
        print(json.dumps({"gate_roofline": gate_saturation_leg(ctx, wl, device)}))
        return
    if only == "ctc_head":
        ctx = Context(device=device)
        print(json.dumps({"ctc_head_gate": ctc_head_leg(ctx, wl, device)}))
        return
    if only == "qformer":
        ctx = Context(device=device)
        print(json.dumps({"qformer_pool": qformer_leg(ctx, wl, device)}))
        return
    if only == "other_configs":
        print(json.dumps({"other_configs": other_configs_leg(args.workload, device, args.steps)}))
        return
    weights = make_model_weights(m, wl.seed, device=device)
    ctx = Context(m, weights, device=device)
    res, step, meta, tau, fl = run_workload(wl, ctx, device, args.steps, args.warmup)
    if only == "ar_fallback":
        print(json.dumps({"ar_fallback": ar_fallback_leg(ctx, wl, meta, tau)}))
        return
    if only == "two_phase":
        print(json.dumps({"two_phase": two_phase_leg(ctx, wl, step, tau, device)}))
        return
    if only == "cpu_baseline":
        print(json.dumps({"cpu_baseline": cpu_baseline(wl, step, weights, meta, args.cpu_budget_rows)}))
        return
    out = {
        "metric": "verified draft tokens/s (gate+verify+accept, whole step)",
        "value": res["verified_draft_tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if m.dtype == "bf16" else "f32",
        "dtype_note": "weights and inputs are stored as bf16; the matrix-core operands are IEEE half (activations rounded to "
                      "11 significant bits instead of bf16's 8, same MFMA rate; weights converted exactly, times a power of two); "
                      "fp32 accumulation, residual stream, softmax and norm statistics" if m.dtype == "bf16" else "all fp32",
        "data": "synthetic",
        "config": {"workload": wl.name, "utterances": wl.B, "verified_utterances": res["verified_utterances"],
                   "decoder_rows": res["decoder_rows"], "draft_tokens": res["draft_tokens"], "ctc_frames": res["ctc_frames"],
                   "V_ctc": wl.V_ctc, "layers": m.n_layers, "d_model": m.d_model, "vocab": m.vocab},
        "utterances_per_s": res["utterances_per_s"],
        "verify_accept_tokens_per_s": res["verify_accept_tokens_per_s"], "verify_accept_ms": res["verify_accept_ms"],
        "gate_pass_rate": res["gate_pass_rate"], "full_accept_rate": res["full_accept_rate"],
        "mean_accepted_prefix_frac": res["mean_accepted_prefix_frac"],
        "verify_roofline": res["verify_roofline"],
    }
    if m.dtype == "bf16":
        dom = dominant_kernel(ctx, step, tau, meta, fl, m, args.steps)
        tr = MEASURED_TRAFFIC.get(wl.name)
        if tr:
            dom["roofline"]["traffic"], dom["roofline"]["traffic_source"] = tr["bytes"], tr["source"]
        out.update(dom)
    else:
        out["roofline"] = dict(res["verify_roofline"], traffic=None)
    hbm = None
    if want("mfma_ceiling") and m.dtype == "bf16":
        tf, ghz = ctx.measure_mfma_ceiling(20000)
        out["mfma_ceiling_this_device"] = {"tflops": tf, "shader_ghz": ghz, "frac_of_nominal_peak": tf / PEAK_MFMA_TFLOPS,
                                           "what": "MFMA-only loop (v_mfma_f32_16x16x32_f16), random f16 operands in registers, 8 wavefronts per CU"}
        out["roofline"]["frac_of_device_ceiling"] = out["roofline"]["achieved"] / tf if tf else None
    if want("hbm_ceiling"):
        big = torch.empty(3 << 30, dtype=torch.uint8, device=device).fill_(1)       # far beyond the memory-side cache
        hbm = ctx.measure_hbm_read(big, 5)
        del big
        out["hbm_read_ceiling_this_device"] = {"gb_per_s": hbm, "frac_of_nominal_peak": hbm / PEAK_HBM_GBS,
                                               "what": "plain streaming read of 3 GiB, one workgroup per CU on its own contiguous share, 8 KB in flight per wavefront"}
    if want("two_phase") and m.dtype == "bf16":
        out["two_phase"] = two_phase_leg(ctx, wl, step, tau, device)
    if want("ar_fallback"):
        out["ar_fallback"] = ar_fallback_leg(ctx, wl, meta, tau)
        if out["ar_fallback"] and hbm:
            out["ar_fallback"]["roofline"]["frac_of_device_ceiling"] = out["ar_fallback"]["roofline"]["achieved"] / hbm
    if want("gate_saturation"):
        out["gate_roofline"] = gate_saturation_leg(ctx, wl, device)
        if hbm:
            out["gate_roofline"]["frac_of_device_ceiling"] = out["gate_roofline"]["achieved"] / hbm
    if want("ctc_head"):
        out["ctc_head_gate"] = ctc_head_leg(ctx, wl, device)
    if want("qformer"):
        out["qformer_pool"] = qformer_leg(ctx, wl, device)
    if want("library_gemm") and m.dtype == "bf16":
        out["library_gemm_reference"] = {"what": "torch.matmul (hipBLASLt) on the same shapes, IEEE half, plain GEMM without "
                                                 "the fused epilogues; compare with projection_tflops", "rows": fl["M"],
                                         **library_gemm_leg(m, fl["M"], device)}
    if want("cpu_baseline"):
        out["cpu_baseline"] = cpu_baseline(wl, step, weights, meta, args.cpu_budget_rows)
    if want("other_configs"):
        del step
        ctx.close()
        del ctx, weights
        torch.cuda.empty_cache()
        out["other_configs"] = other_configs_leg(args.workload, device, args.steps)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
