"""Two-phase batched decoding schedule of Sec. 3.2 around the library's calls (host-side policy only).

The paper sorts utterances by length, cuts them into batches under a token budget (50K tokens), batches the
CTC + LLM-verification pass separately from the auto-regressive fallback pass, and parks the acoustic embeddings
in host memory between the two.  `TwoPhaseDecoder.run` is that schedule:

  gate      ctc_gate over the whole batch (a streaming kernel without activations: no reason to cut it up)
  phase 1   verification bins planned with ssd_plan_batches on S + P + U of the utterances that failed the gate;
            per bin: ssd_select_unconfident -> verify_forward[_kv] -> accept_prefix
  between   mode "offload" (the paper's): the acoustic embeddings g of the rejected utterances are copied to pinned
            host memory and nothing else of phase 1 is kept; mode "resident": the K/V cache of phase 1 stays in HBM
            (what 288 GB make possible: a 50K-token batch of the 1B-class decoder is 4.9 GB of keys and values)
  phase 2   fallback bins planned on context length + steps of the rejected utterances; per bin, "offload" reloads g,
            re-runs the prompt [g; prompt; accepted prefix + the rejected token] with verify_forward_kv (whose greedy
            token at the rejected position is the first fallback token) and then ar_fallback; "resident" calls
            ar_fallback on the cached rows directly.

Everything numeric happens inside the library; this module only decides what goes into which call.  Copies between
device and pinned host memory are plain memcpys issued through torch on the context's stream.
"""
from typing import Optional

import numpy as np
import torch

from .binding import Context, plan_batches


class TwoPhaseDecoder:
    def __init__(self, ctx: Context, wl, logits: torch.Tensor, cu_frames, ctc_to_llm: torch.Tensor,
                 speech_all: torch.Tensor, cu_speech_all, prompt_all: torch.Tensor, cu_prompt_all,
                 budget: int = 50000, mode: str = "resident", n_steps: int = 8):
        assert mode in ("offload", "resident")
        self.ctx, self.wl, self.mode, self.budget, self.n_steps = ctx, wl, mode, int(budget), int(n_steps)
        self.logits, self.table = logits, ctc_to_llm
        self.cu_frames = np.ascontiguousarray(cu_frames, dtype=np.int32)
        self.speech_all, self.prompt_all = speech_all, prompt_all
        self.cu_s = np.ascontiguousarray(cu_speech_all, dtype=np.int32)
        self.cu_p = np.ascontiguousarray(cu_prompt_all, dtype=np.int32)
        self.B = len(self.cu_frames) - 1
        self.S, self.P, self.T = np.diff(self.cu_s), np.diff(self.cu_p), np.diff(self.cu_frames)
        dev, m = ctx.device, ctx.cfg
        n_frames, nS, nP = int(self.cu_frames[-1]), int(self.cu_s[-1]), int(self.cu_p[-1])
        # the largest bin is bounded by the budget, or by the longest utterance when that alone exceeds it
        longest = int((self.S + self.P + self.T).max()) + self.n_steps + 2
        cap = min(max(self.budget, longest), nS + nP + n_frames + self.B * (self.n_steps + 2))
        ctx.reserve(max_frames=n_frames, max_tokens=cap, max_verify_rows=min(cap, n_frames), max_utts=self.B,
                    ar_utts=self.B, ar_steps=self.n_steps)
        self.sel_buf = {"speech": torch.empty((min(cap, nS), m.d_model), dtype=speech_all.dtype, device=dev),
                        "prompt": torch.empty(min(cap, nP), dtype=torch.int32, device=dev),
                        "draft_ids": torch.empty(min(cap, n_frames), dtype=torch.int32, device=dev)}
        self.hv_buf = torch.empty((min(cap, n_frames), m.d_model), dtype=ctx.act_dtype, device=dev)
        # likelihoods and greedy tokens of every draft position of the batch, bins one after the other
        self.logp_all = torch.empty(n_frames, dtype=torch.float32, device=dev)
        self.greedy_all = torch.empty(n_frames, dtype=torch.int32, device=dev)
        self.gate_out = None
        # K/V slots: every verified utterance keeps its rows (resident), or one fallback bin at a time (offload)
        slots = (nS + nP + n_frames + self.B * (self.n_steps + 2)) if mode == "resident" else cap + self.B * (self.n_steps + 2)
        ctx.set_kv_cache(int(slots))
        self.kv_slots = int(slots)
        self.host_g: Optional[torch.Tensor] = None       # pinned staging for the acoustic embeddings (offload mode)
        if mode == "offload":
            self.host_g = torch.empty((nS, m.d_model), dtype=speech_all.dtype, pin_memory=True)
            self.dev_g = torch.empty((min(cap, nS), m.d_model), dtype=speech_all.dtype, device=dev)

    def _bins(self, lengths):
        return plan_batches(lengths, self.budget, padded=False) if len(lengths) else []

    def run(self, tau_slm: float) -> dict:
        ctx, wl, n_steps = self.ctx, self.wl, self.n_steps
        # ---- gate (Sec. 2.1) over everything
        g = ctx.ctc_gate(self.logits, self.cu_frames, wl.blank_id, wl.tau_ctc, out=self.gate_out)
        self.gate_out = g
        gate_pass = g["gate_pass"].cpu().numpy().astype(bool)
        draft_len = g["draft_len"].cpu().numpy()
        fail = np.flatnonzero(~gate_pass)
        res = {"gate_pass": gate_pass, "draft_len": draft_len, "accept_len": np.full(self.B, -1, np.int32),
               "tokens": {}, "verify_bins": 0, "fallback_bins": 0, "rejected": 0, "offloaded_bytes": 0}
        if len(fail) == 0:
            return res
        # ---- phase 1: verification bins (Sec. 2.2), longest first under the token budget
        n_rows = (self.S + self.P + draft_len)[fail]
        bins = [fail[b] for b in self._bins(n_rows)]
        res["verify_bins"] = len(bins)
        kv_next = 0
        kv_start = np.zeros(self.B, np.int32)
        pending = []
        off = 0                                                # draft positions handed out so far
        goff = np.zeros(self.B, np.int64)                      # where an utterance's draft starts in logp_all / greedy_all
        for utts in bins:
            sel = ctx.select_unconfident(utts, self.cu_frames, draft_len, g["draft_ctc"], self.table, self.speech_all,
                                         self.cu_s, self.prompt_all, self.cu_p, out=self.sel_buf)
            Mv = int(sel["cu_draft"][-1])
            ks = None
            if self.mode == "resident":
                cap = (self.S + self.P + draft_len)[utts] + n_steps + 2
                ks = (kv_next + np.concatenate([[0], np.cumsum(cap)[:-1]])).astype(np.int32)
                kv_start[utts] = ks
                kv_next += int(cap.sum())
            hv = ctx.verify_forward(sel["speech"], sel["cu_speech"], sel["prompt"], sel["cu_prompt"], sel["draft_ids"],
                                    sel["cu_draft"], out=self.hv_buf[:Mv], kv_start=ks)
            acc = ctx.accept_prefix(hv, sel["draft_ids"], sel["cu_draft"], tau_slm,
                                    out={"draft_logp": self.logp_all[off:off + Mv], "greedy_tok": self.greedy_all[off:off + Mv],
                                         "accept_len": torch.empty(len(utts), dtype=torch.int32, device=ctx.device),
                                         "all_accepted": torch.empty(len(utts), dtype=torch.uint8, device=ctx.device)})
            goff[utts] = off + sel["cu_draft"][:-1]
            off += Mv
            pending.append((utts, acc))
        # one wait for the whole phase: prefix lengths decide who goes on
        for utts, acc in pending:
            res["accept_len"][utts] = acc["accept_len"].cpu().numpy()
        rej = np.array([b for b in fail if res["accept_len"][b] < draft_len[b]], dtype=np.int64)
        res["rejected"] = len(rej)
        if len(rej) == 0:
            return res
        A = res["accept_len"]
        # ---- between the phases
        if self.mode == "offload":
            with torch.cuda.stream(ctx.stream):
                for b in rej:                                  # g of the rejected utterances -> pinned host memory
                    lo, hi = int(self.cu_s[b]), int(self.cu_s[b + 1])
                    self.host_g[lo:hi].copy_(self.speech_all[lo:hi], non_blocking=True)
                    res["offloaded_bytes"] += (hi - lo) * self.speech_all.shape[1] * self.speech_all.element_size()
            ctx.stream.synchronize()                           # phase 1 is over; nothing of it stays on the device
        # ---- phase 2: fallback bins (Sec. 2.3) on context length + the tokens to come
        ctx_len_all = (self.S + self.P + A).astype(np.int32)
        fb_bins = [rej[b] for b in self._bins((ctx_len_all[rej] + n_steps + 2).astype(np.int32))]
        res["fallback_bins"] = len(fb_bins)
        outs = []
        for utts in fb_bins:
            if self.mode == "resident":
                # the first fallback token is the model's own choice at the first rejected position
                first = ctx.gather_i32(self.greedy_all, goff[utts] + A[utts])
                ks, cl = kv_start[utts], ctx_len_all[utts]
            else:
                # reload g, then re-run [g; prompt; accepted prefix + the rejected token] with the K/V cache on
                S_u = self.S[utts]
                cu_su = np.concatenate([[0], np.cumsum(S_u)]).astype(np.int32)
                with torch.cuda.stream(ctx.stream):
                    for k, b in enumerate(utts):
                        self.dev_g[int(cu_su[k]):int(cu_su[k + 1])].copy_(self.host_g[int(self.cu_s[b]):int(self.cu_s[b + 1])], non_blocking=True)
                re_len = draft_len.copy()
                re_len[utts] = A[utts] + 1
                sel = ctx.select_unconfident(utts, self.cu_frames, re_len, g["draft_ctc"], self.table, None,
                                             np.zeros(self.B + 1, np.int32), self.prompt_all, self.cu_p,
                                             out={"speech": self.sel_buf["speech"][:0], "prompt": self.sel_buf["prompt"],
                                                  "draft_ids": self.sel_buf["draft_ids"]}, d_model=int(self.speech_all.shape[1]),
                                             dtype=self.speech_all.dtype)
                cap = (self.S + self.P + A)[utts] + n_steps + 2
                ks = np.concatenate([[0], np.cumsum(cap)[:-1]]).astype(np.int32)
                cl = ctx_len_all[utts]
                Mv = int(sel["cu_draft"][-1])
                hv = ctx.verify_forward(self.dev_g[:int(cu_su[-1])], cu_su, sel["prompt"], sel["cu_prompt"], sel["draft_ids"],
                                        sel["cu_draft"], out=self.hv_buf[:Mv], kv_start=ks)
                acc = ctx.accept_prefix(hv, sel["draft_ids"], sel["cu_draft"], tau_slm, want_greedy=True)
                first = ctx.gather_i32(acc["greedy_tok"], sel["cu_draft"][1:] - 1)
            toks = ctx.ar_fallback(ks, cl, first, n_steps)
            outs.append((utts, first, toks))
        for utts, first, toks in outs:
            f, t = first.cpu().numpy(), toks.cpu().numpy()
            for k, b in enumerate(utts):
                res["tokens"][int(b)] = np.concatenate([[f[k]], t[:, k]]).astype(np.int32)
        return res
