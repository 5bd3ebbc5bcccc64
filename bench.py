#!/usr/bin/env python3
"""Benchmark of the gate -> verify -> accept hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]

A step is one pass of the whole path over one synthetic batch that is already resident in HBM:
ctc_gate -> (read gate flags and draft lengths, map CTC ids to LLM ids: the caller's glue) ->
verify_forward -> accept_prefix.  Prints ONE JSON line.
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

# Memory traffic of the dominant kernel per launch, from two rocprofv3 --pmc runs of this file
# (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch), each scaled by what the same counter reads for a
# plain 1 GiB device copy (`--copy-reference`): FETCH_SIZE reads 524301 for 1048576 KiB (factor 2.0),
# WRITE_SIZE reads 1048576 (factor 1.0).  See profiles/pmc_traffic_gemm_gate_up_cfg3.md.
MEASURED_TRAFFIC_BYTES = {
    "cfg3_1b_ragged64": (354061.6 * 2.0 + 84440.0 * 1.0) * 1024.0,      # a full layer (5144 rows)
}


class Step:
    """Everything one step needs, prepared once; `run()` enqueues one step and returns its outputs."""

    def __init__(self, wl, ctx, device):
        from paper_2603_11243_amd.binding import Context  # noqa: F401
        self.wl, self.ctx = wl, ctx
        self.cb = make_ctc_batch(wl)
        self.logits = self.cb.logits.to(device)
        self.table = torch.from_numpy(make_ctc_to_llm_map(wl)).to(device)
        self.cu_frames = self.cb.cu_frames
        B, n_frames = wl.B, int(self.cu_frames[-1])
        # Inputs of the verify pass exist for every utterance; a step uses those of the utterances
        # that fail the gate.  Speech rows: round(6 * seconds) (or the fixed count), prompt ids random.
        self.vi_all = make_verify_inputs(wl, self.cb.seconds, [np.zeros(0, np.int32)] * B, device=device)
        self.prompt_ids = torch.from_numpy(self.vi_all.prompt_ids).to(device)
        self.gate_out = None
        max_tok = int(self.vi_all.cu_speech[-1] + self.vi_all.cu_prompt[-1]) + n_frames      # a draft is at most T tokens
        ctx.reserve(max_frames=n_frames, max_tokens=max_tok, max_verify_rows=n_frames, max_utts=B)
        self.device = device
        self.frame_off = torch.from_numpy(self.cu_frames[:-1].astype(np.int64)).to(device)

    def run(self, tau_slm):
        wl, ctx, vi = self.wl, self.ctx, self.vi_all
        g = ctx.ctc_gate(self.logits, self.cu_frames, wl.blank_id, wl.tau_ctc, out=self.gate_out)
        self.gate_out = g
        # ---- caller's glue: which utterances go on, how long their drafts are, CTC id -> LLM id
        flags = torch.stack([g["gate_pass"].to(torch.int32), g["draft_len"]]).cpu().numpy()   # one D2H sync
        fail = np.flatnonzero(flags[0] == 0)
        if len(fail) == 0:
            return g, None, None, 0
        U = flags[1][fail]
        cu_d = np.zeros(len(fail) + 1, np.int32); cu_d[1:] = np.cumsum(U)
        S = np.diff(vi.cu_speech)[fail]; P = np.diff(vi.cu_prompt)[fail]
        cu_s = np.zeros(len(fail) + 1, np.int32); cu_s[1:] = np.cumsum(S)
        cu_p = np.zeros(len(fail) + 1, np.int32); cu_p[1:] = np.cumsum(P)
        # gather index of the draft tokens inside draft_ctc, and of the speech / prompt rows
        starts = self.cu_frames[:-1][fail].astype(np.int64)
        idx = np.repeat(starts - cu_d[:-1], U) + np.arange(int(cu_d[-1]))
        draft_ids = self.table[g["draft_ctc"][torch.from_numpy(idx).to(self.device)].long()].to(torch.int32)
        if len(fail) == wl.B:
            speech, prompt = vi.speech_emb, self.prompt_ids
        else:
            sidx = np.repeat(vi.cu_speech[:-1][fail].astype(np.int64) - cu_s[:-1], S) + np.arange(int(cu_s[-1]))
            pidx = np.repeat(vi.cu_prompt[:-1][fail].astype(np.int64) - cu_p[:-1], P) + np.arange(int(cu_p[-1]))
            speech = vi.speech_emb[torch.from_numpy(sidx).to(self.device)]
            prompt = self.prompt_ids[torch.from_numpy(pidx).to(self.device)]
        hv = ctx.verify_forward(speech, cu_s, prompt, cu_p, draft_ids, cu_d)
        acc = ctx.accept_prefix(hv, draft_ids, cu_d, tau_slm)
        meta = {"fail": fail, "cu_s": cu_s, "cu_p": cu_p, "cu_d": cu_d, "speech": speech, "prompt": prompt,
                "draft_ids": draft_ids}
        return g, acc, meta, int(cu_d[-1])


def tau_for(wl, q=1.9):
    s = 0.02 * np.sqrt(wl.model.d_model)
    return float(np.exp(-np.log(wl.model.vocab) - s * s / 2 - q * s))


def cpu_baseline(wl, step, weights, meta, budget_tokens):
    """The oracle, as it stands, on this machine's host cores, over a bounded sample of the same batch."""
    from oracle import ssd_oracle as O
    import threadpoolctl
    cores = max((p["num_threads"] for p in threadpoolctl.threadpool_info() if p.get("user_api") == "blas"), default=1)
    fail = meta["fail"]
    lens = np.diff(meta["cu_s"]) + np.diff(meta["cu_p"]) + np.diff(meta["cu_d"])
    order = np.argsort(-lens)
    pick, tok = [], 0
    for k in order[len(order) // 2:]:                       # start from median-length utterances
        if tok + lens[k] > budget_tokens and pick:
            break
        pick.append(int(k)); tok += int(lens[k])
    # host copies, widened outside the timed region (the oracle's arithmetic is what is timed)
    w64 = {"embed": weights["embed"].double().cpu(), "lm_head": weights["lm_head"].double().cpu(),
           "norm_final": weights["norm_final"].double().cpu(),
           "layers": [{k: v.double().cpu() for k, v in L.items()} for L in weights["layers"]]}
    cu = lambda a: np.concatenate([[0], np.cumsum(a)]).astype(np.int32)
    sp = torch.cat([meta["speech"][meta["cu_s"][k]:meta["cu_s"][k + 1]] for k in pick]).double().cpu()
    pr = np.concatenate([meta["prompt"][meta["cu_p"][k]:meta["cu_p"][k + 1]].cpu().numpy() for k in pick])
    dr = np.concatenate([meta["draft_ids"][meta["cu_d"][k]:meta["cu_d"][k + 1]].cpu().numpy() for k in pick])
    cs, cp, cd = (cu(np.diff(meta[n])[pick]) for n in ("cu_s", "cu_p", "cu_d"))
    utt = fail[pick]
    rows = np.concatenate([np.arange(step.cu_frames[b], step.cu_frames[b + 1]) for b in utt])
    z = step.cb.logits[rows].float().numpy()
    cuf = cu([step.cu_frames[b + 1] - step.cu_frames[b] for b in utt])
    t0 = time.perf_counter()
    O.ctc_gate(z, cuf, wl.blank_id, wl.tau_ctc)
    lp = O.draft_logp(w64, wl.model, sp, cs, pr, cp, dr, cd)
    for x in lp:
        O.accept_prefix(x, tau_for(wl))
    dt = time.perf_counter() - t0
    n_draft = int(cd[-1])
    return {"value": n_draft / dt, "unit": "verified draft tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{len(pick)} of {len(fail)} verified utterances ({n_draft} draft tokens, {tok} decoder rows), "
                      f"gate+verify+accept in float64 numpy, {dt:.1f} s",
            "utterances_per_s": len(pick) / dt}


def gate_roofline(ctx, wl, device):
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
    return {"bound": "hbm", "kernel": "ctc_gate (frames kernel + per-utterance kernel)", "achieved": gbs,
            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS, "avg_call_ms": ms / n,
            "frames": n_rows, "V_ctc": V, "storage": str(dt).replace("torch.", ""), "bytes_per_frame": V * z.element_size() + 12}


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
                         "flops_per_call": flops, "note": "348 symbols occupy 512 MFMA columns: 68 % of the issued flops are algorithmic"},
            "bytes_per_frame": {"fused": d_enc * 2 + 16 * ((V + 63) // 64) * 2 + 12, "unfused": d_enc * 2 + 2 * Vs * 2 + 12}}


def single_utterance_leg(ctx, wl, device, steps=50):
    """The B=1 configuration of the same decoder (one 10 s utterance, ~108 decoder rows): a step is bound by
    streaming every weight once, so it is graded against HBM bandwidth.  Same context and weights."""
    name = {"cfg3_1b_ragged64": "cfg2_1b_b1"}.get(wl.name)
    if name is None or WORKLOADS[name].model != wl.model:
        return None
    w1 = WORKLOADS[name]
    step = Step(w1, ctx, device)
    tau = tau_for(w1)
    for _ in range(5):
        g, acc, meta, n_draft = step.run(tau)
    torch.cuda.synchronize()
    if acc is None:
        return None
    t0 = time.perf_counter()
    for _ in range(steps):
        step.run(tau)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    m = w1.model
    M = int(meta["cu_s"][-1] + meta["cu_p"][-1] + meta["cu_d"][-1])
    weight_bytes = 2.0 * (m.n_layers * m.params_per_layer() + m.vocab * m.d_model)
    gbs = weight_bytes / (ms * 1e-3) / 1e9
    return {"workload": name, "decoder_rows": M, "draft_tokens": n_draft, "ms_per_step": ms,
            "verified_draft_tokens_per_s": n_draft / (ms * 1e-3),
            "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                         "algorithmic_bytes_per_step": weight_bytes}}


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
    weight_bytes = 2.0 * (m.n_layers * m.params_per_layer() + m.vocab * m.d_model)
    gbs = weight_bytes / (step_ms * 1e-3) / 1e9
    return {"rejected_utterances": int(len(rej)), "steps": n_steps, "ms_per_step": step_ms,
            "tokens_per_s": len(rej) / (step_ms * 1e-3),
            "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                         "algorithmic_bytes_per_step": weight_bytes}}


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3_1b_ragged64", choices=list(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget-tokens", type=int, default=3000)
    ap.add_argument("--main-only", action="store_true",
                    help="skip the side legs (MFMA ceiling, AR fallback, gate saturation, CTC head): for counter runs")
    ap.add_argument("--copy-reference", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy five times (scale reference for --pmc counters)")
    ap.add_argument("--mfma-ceiling-only", action="store_true",
                    help="only run the MFMA-only ceiling kernel (a kernel whose matrix cores never idle: the 100 % mark "
                         "for the MFMA-busy counters of a --pmc run)")
    args = ap.parse_args()
    if args.mfma_ceiling_only:
        from paper_2603_11243_amd.binding import Context
        wl = WORKLOADS["cfg1_tiny_f32"]
        ctx = Context(wl.model, make_model_weights(wl.model, wl.seed, device=torch.device("cuda:0")), device=torch.device("cuda:0"))
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
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on ONE GPU (utterance-sharded data parallelism needs no collectives and is "
              "not built); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    from paper_2603_11243_amd.binding import Context
    device = torch.device("cuda:0")
    wl = WORKLOADS[args.workload]
    m = wl.model
    weights = make_model_weights(m, wl.seed, device=device)
    ctx = Context(m, weights, device=device)
    step = Step(wl, ctx, device)
    tau = tau_for(wl)

    for _ in range(max(args.warmup, 1)):
        g, acc, meta, n_draft = step.run(tau)
    torch.cuda.synchronize()
    ctx.profile_select("gemm_gate_up")              # time the dominant kernel with HIP events, live
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        g, acc, meta, n_draft = step.run(tau)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    dom_ms, dom_n = ctx.profile_read()["gemm_gate_up"]

    # per-class breakdown in one extra, untimed step
    ctx.profile_select(-1)
    step.run(tau)
    breakdown = {k: round(v[0], 4) for k, v in ctx.profile_read().items()}
    ctx.profile_select(-2)
    # verify+accept alone (metric (i) of the workload definition)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        hv = ctx.verify_forward(meta["speech"], meta["cu_s"], meta["prompt"], meta["cu_p"], meta["draft_ids"], meta["cu_d"])
        ctx.accept_prefix(hv, meta["draft_ids"], meta["cu_d"], tau)
    torch.cuda.synchronize()
    dt_va = time.perf_counter() - t1

    ms_per_step = dt / args.steps * 1e3
    M = int(meta["cu_s"][-1] + meta["cu_p"][-1] + meta["cu_d"][-1])
    Bv = len(meta["fail"])
    # rows per launch: M in every layer but the last, where only the Mv verification rows continue after
    # attention (Eq. 5 scores nothing else); the average launch is priced with the average row count
    Mv = int(meta["cu_d"][-1])
    L = m.n_layers
    rows_avg = ((L - 1) * M + Mv) / L
    gate_up_flops = 2.0 * rows_avg * m.d_model * 2 * m.d_ff
    avg_ms = dom_ms / max(dom_n, 1)
    achieved = gate_up_flops / (avg_ms * 1e-3) / 1e12 if dom_n else 0.0
    gemm_ms = sum(breakdown[k] for k in ("gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down"))
    qkv_params = m.d_model * (m.d_q + 2 * m.d_kv)
    step_gemm_flops = 2.0 * (L * M * qkv_params + L * rows_avg * (m.params_per_layer() - qkv_params))
    acc_len = acc["accept_len"].cpu().numpy()
    out = {
        "metric": "verified draft tokens/s (gate+verify+accept, whole step)",
        "value": n_draft / (dt / args.steps), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if m.dtype == "bf16" else "f32",
        "dtype_note": "matrix-core operands are IEEE half (weights stored as bf16 are converted exactly, times a power of two); "
                      "fp32 accumulation, residual stream, softmax and norm statistics" if m.dtype == "bf16" else "all fp32",
        "data": "synthetic",
        "config": {"workload": wl.name, "utterances": wl.B, "verified_utterances": Bv, "decoder_rows": M,
                   "draft_tokens": n_draft, "ctc_frames": int(step.cu_frames[-1]), "V_ctc": wl.V_ctc,
                   "layers": m.n_layers, "d_model": m.d_model, "vocab": m.vocab},
        "utterances_per_s": wl.B / (dt / args.steps),
        "verify_accept_tokens_per_s": n_draft / (dt_va / args.steps),
        "gate_pass_rate": float(g["gate_pass"].float().mean().cpu()),
        "full_accept_rate": float(acc["all_accepted"].float().mean().cpu()),
        "mean_accepted_prefix_frac": float(np.mean(acc_len / np.maximum(np.diff(meta["cu_d"]), 1))),
        "roofline": {"bound": "mfma", "kernel": "gemm_mfma16_kernel<EpiSwiglu> (gate/up projection + SiLU*mul)",
                     "achieved": achieved, "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_MFMA_TFLOPS, "traffic": MEASURED_TRAFFIC_BYTES.get(wl.name),
                     "traffic_unit": "bytes per launch (L2<->fabric, incl. Infinity Cache hits)",
                     "algorithmic_bytes": 2.0 * (rows_avg * m.d_model + 2 * m.d_ff * m.d_model + rows_avg * m.d_ff),
                     "rows_per_launch": {"layers_before_last": M, "last_layer": Mv, "average": rows_avg},
                     "avg_launch_ms": avg_ms, "launches_timed": dom_n, "flops_per_launch": gate_up_flops},
        "breakdown_ms_per_step": breakdown,
        "all_projection_gemms": {"tflops": step_gemm_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms else None,
                                 "frac_of_peak": step_gemm_flops / (gemm_ms * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS if gemm_ms else None},
    }
    # per projection: flops of a step over the HIP-event time of that class in the breakdown step
    per_gemm_flops = {"gemm_qkv": 2.0 * L * M * qkv_params, "gemm_o": 2.0 * L * rows_avg * m.d_model * m.d_q,
                      "gemm_gate_up": 2.0 * L * rows_avg * m.d_model * 2 * m.d_ff, "gemm_down": 2.0 * L * rows_avg * m.d_model * m.d_ff}
    out["projection_tflops"] = {k: (f / (breakdown[k] * 1e-3) / 1e12 if breakdown.get(k) else None) for k, f in per_gemm_flops.items()}
    # accept_prefix: LM head fused with the log-softmax and the gather (+ finalize and prefix scan), HIP-event time
    # of the class in the breakdown step.  MFMA bound above about 310 rows, weight streaming below.
    if breakdown.get("lmhead_accept"):
        t_acc = breakdown["lmhead_accept"] * 1e-3
        acc_flops = 2.0 * Mv * m.vocab * m.d_model
        acc_bytes = 2.0 * (m.vocab * m.d_model + Mv * m.d_model) + 4.0 * Mv
        if Mv > 310:
            out["accept_roofline"] = {"bound": "mfma", "achieved": acc_flops / t_acc / 1e12, "peak": PEAK_MFMA_TFLOPS,
                                      "unit": "TFLOP/s", "frac": acc_flops / t_acc / 1e12 / PEAK_MFMA_TFLOPS,
                                      "rows": Mv, "ms": breakdown["lmhead_accept"],
                                      "logit_bytes_never_written": 4.0 * Mv * m.vocab}
        else:
            out["accept_roofline"] = {"bound": "hbm", "achieved": acc_bytes / t_acc / 1e9, "peak": PEAK_HBM_GBS,
                                      "unit": "GB/s", "frac": acc_bytes / t_acc / 1e9 / PEAK_HBM_GBS,
                                      "rows": Mv, "ms": breakdown["lmhead_accept"],
                                      "logit_bytes_never_written": 4.0 * Mv * m.vocab}
    if not args.main_only:
        tf, ghz = ctx.measure_mfma_ceiling(20000)
        out["mfma_ceiling_this_device"] = {"tflops": tf, "shader_ghz": ghz, "frac_of_nominal_peak": tf / PEAK_MFMA_TFLOPS,
                                           "what": "MFMA-only loop (v_mfma_f32_16x16x32_f16), random f16 operands in registers, 8 wavefronts per CU"}
        out["roofline"]["frac_of_device_ceiling"] = achieved / tf if tf else None
        big = torch.empty(3 << 30, dtype=torch.uint8, device=device).fill_(1)       # far beyond the memory-side cache
        hbm = ctx.measure_hbm_read(big, 5)
        del big
        out["hbm_read_ceiling_this_device"] = {"gb_per_s": hbm, "frac_of_nominal_peak": hbm / PEAK_HBM_GBS,
                                               "what": "plain streaming read of 3 GiB, one workgroup per CU on its own contiguous share, 8 KB in flight per wavefront"}
        out["ar_fallback"] = ar_fallback_leg(ctx, wl, meta, tau)
        if out["ar_fallback"]:
            out["ar_fallback"]["roofline"]["frac_of_device_ceiling"] = out["ar_fallback"]["roofline"]["achieved"] / hbm
        out["gate_roofline"] = gate_roofline(ctx, wl, device)
        out["gate_roofline"]["frac_of_device_ceiling"] = out["gate_roofline"]["achieved"] / hbm
        out["ctc_head_gate"] = ctc_head_leg(ctx, wl, device)
        out["single_utterance"] = single_utterance_leg(ctx, wl, device)
        if m.dtype == "bf16":
            out["library_gemm_reference"] = {"what": "torch.matmul (hipBLASLt) on the same shapes, IEEE half, plain GEMM without "
                                                     "the fused epilogues; compare with projection_tflops", "rows": M,
                                             **library_gemm_leg(m, M, device)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, step, weights, meta, args.cpu_budget_tokens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
