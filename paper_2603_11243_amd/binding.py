"""ctypes binding of the C ABI in include/ssd.h: argument marshalling only.

Torch is used for device memory (tensors own the buffers, `data_ptr()` is what crosses the ABI)
and for the stream handle.  Every computation happens inside libssd.so.
"""
import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libssd.so")

SSD_F32, SSD_BF16 = 0, 1
_DTYPE_CODE = {torch.float32: SSD_F32, torch.bfloat16: SSD_BF16}
_STATUS = {0: "SSD_OK", -1: "SSD_EINVAL", -2: "SSD_ESHAPE", -3: "SSD_EWORKSPACE", -4: "SSD_EHIP",
           -5: "SSD_EUNSUPPORTED"}

EXPORTS = ["ssd_create", "ssd_destroy", "ssd_workspace_bytes", "ssd_set_workspace", "ssd_last_error",
           "ssd_profile_select", "ssd_profile_read", "ssd_measure_mfma_ceiling", "ssd_measure_hbm_read", "ctc_gate", "verify_forward", "accept_prefix",
           "verify_forward_kv", "ssd_kv_cache_bytes", "ssd_set_kv_cache", "ssd_ar_workspace_bytes", "ar_fallback",
           "ssd_gate_grid", "ssd_accept_grid", "ssd_plan_batches", "ssd_set_ctc_head", "ctc_head_gate", "ssd_device_flags",
           "ctc_gate_noalloc", "ssd_inexact_weights", "ssd_select_unconfident", "ssd_gather_i32", "ssd_set_qformer", "qformer_pool"]

PROF_OFF, PROF_ALL = -2, -1
PROF_CLASSES = ["gate", "gemm_qkv", "attention", "gemm_o", "gemm_gate_up", "gemm_down", "lmhead_accept", "other",
                "ar_fallback", "ctc_head_gate", "qformer_pool"]


class SsdError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"{_STATUS.get(code, code)}: {msg}")
        self.code = code


class ModelCfgC(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ff", C.c_int32), ("vocab", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("dtype", C.c_int32),
                ("max_positions", C.c_int32), ("operand", C.c_int32)]


class WeightsC(C.Structure):
    _fields_ = [("embed", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down",
                                                      "norm_attn", "norm_mlp")] + \
               [("norm_final", C.c_void_p), ("lm_head", C.c_void_p)]


def load_library() -> C.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2603_11243_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int, C.c_int64, C.c_float
    lib.ssd_create.argtypes = [C.POINTER(vp), C.POINTER(ModelCfgC), C.POINTER(WeightsC), vp]
    lib.ssd_create.restype = i32
    lib.ssd_destroy.argtypes = [vp]
    lib.ssd_destroy.restype = None
    lib.ssd_workspace_bytes.argtypes = [vp, i64, i64, i64, i64]
    lib.ssd_workspace_bytes.restype = C.c_size_t
    lib.ssd_set_workspace.argtypes = [vp, vp, C.c_size_t]
    lib.ssd_set_workspace.restype = i32
    lib.ssd_last_error.argtypes = [vp]
    lib.ssd_last_error.restype = C.c_char_p
    lib.ssd_profile_select.argtypes = [vp, i32]
    lib.ssd_profile_select.restype = i32
    lib.ssd_profile_read.argtypes = [vp, vp, vp]
    lib.ssd_profile_read.restype = i32
    lib.ssd_measure_mfma_ceiling.argtypes = [vp, i32, vp, vp]
    lib.ssd_measure_mfma_ceiling.restype = i32
    lib.ssd_measure_hbm_read.argtypes = [vp, vp, C.c_size_t, i32, vp]
    lib.ssd_measure_hbm_read.restype = i32
    lib.ctc_gate.argtypes = [vp, vp, i32, vp, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp]
    lib.ctc_gate.restype = i32
    lib.verify_forward.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, vp]
    lib.verify_forward.restype = i32
    lib.accept_prefix.argtypes = [vp, vp, vp, vp, i32, f32, vp, vp, vp, vp]
    lib.accept_prefix.restype = i32
    lib.verify_forward_kv.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, vp, vp]
    lib.verify_forward_kv.restype = i32
    lib.ssd_kv_cache_bytes.argtypes = [vp, i64]
    lib.ssd_kv_cache_bytes.restype = C.c_size_t
    lib.ssd_set_kv_cache.argtypes = [vp, vp, C.c_size_t, i64]
    lib.ssd_set_kv_cache.restype = i32
    lib.ssd_ar_workspace_bytes.argtypes = [vp, i32, i32]
    lib.ssd_ar_workspace_bytes.restype = C.c_size_t
    lib.ar_fallback.argtypes = [vp, i32, vp, vp, vp, i32, vp]
    lib.ar_fallback.restype = i32
    lib.ssd_gate_grid.argtypes = [vp, vp, i32, vp, i32, vp]
    lib.ssd_gate_grid.restype = i32
    lib.ssd_accept_grid.argtypes = [vp, vp, vp, i32, vp, i32, vp, vp]
    lib.ssd_accept_grid.restype = i32
    lib.ssd_plan_batches.argtypes = [vp, i32, i64, i32, vp, vp, vp]
    lib.ssd_plan_batches.restype = i32
    lib.ssd_device_flags.argtypes = [vp, vp]
    lib.ssd_device_flags.restype = i32
    lib.ssd_set_ctc_head.argtypes = [vp, vp, vp, i32, i32]
    lib.ssd_set_ctc_head.restype = i32
    lib.ctc_head_gate.argtypes = [vp, vp, vp, i32, i32, f32, vp, vp, vp, vp, vp, vp]
    lib.ctc_head_gate.restype = i32
    lib.ctc_gate_noalloc.argtypes = [vp, vp, i32, vp, i32, i64, i32, i32, f32, vp, vp, vp, vp, C.c_char_p, C.c_size_t]
    lib.ctc_gate_noalloc.restype = i32
    lib.ssd_select_unconfident.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.ssd_select_unconfident.restype = i32
    lib.ssd_set_qformer.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32]
    lib.ssd_set_qformer.restype = i32
    lib.qformer_pool.argtypes = [vp, vp, vp, i32, vp, vp]
    lib.qformer_pool.restype = i32
    lib.ssd_gather_i32.argtypes = [vp, vp, vp, i32, vp]
    lib.ssd_gather_i32.restype = i32
    lib.ssd_inexact_weights.argtypes = [vp]
    lib.ssd_inexact_weights.restype = i64
    return lib


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = load_library()
    return _lib


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous()
    return C.c_void_p(t.data_ptr())


def _host_i32(a: Sequence[int]) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


class Context:
    """Owns one ssd_ctx.  `weights` is the dict layout of workloads.make_model_weights (device tensors)."""

    def __init__(self, model_cfg=None, weights: Optional[dict] = None, device="cuda:0", stream=None,
                 max_positions: int = 1024, operand: str = "f16"):
        self._lib = lib()
        self.device = torch.device(device)
        self.cfg = model_cfg
        self._keep = []               # tensors whose storage the library reads in place
        self._ws = None
        self._h = C.c_void_p()
        torch.cuda.set_device(self.device)
        st = stream if stream is not None else torch.cuda.current_stream(self.device)
        self.stream = st
        cfg_p, w_p = None, None
        if model_cfg is not None:
            m = model_cfg
            self.dtype = {"bf16": torch.bfloat16, "f32": torch.float32}[m.dtype]
            # h_verify is an activation buffer between verify_forward and accept_prefix: the MFMA operand type for
            # bf16-stored models (IEEE half by default, bfloat16 with operand="bf16"), fp32 otherwise
            self.operand = operand
            self.act_dtype = torch.float32 if m.dtype == "f32" else {"f16": torch.float16, "bf16": torch.bfloat16}[operand]
            cfg_c = ModelCfgC(m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.d_ff, m.vocab,
                              m.rms_eps, m.rope_theta, _DTYPE_CODE[self.dtype], max_positions,
                              {"f16": 0, "bf16": 1}[operand])
            w_c = WeightsC()

            def dev(t):
                t = t.to(self.device).contiguous()
                assert t.dtype == self.dtype
                self._keep.append(t)
                return t.data_ptr()

            w_c.embed = dev(weights["embed"])
            w_c.lm_head = dev(weights["lm_head"])
            w_c.norm_final = dev(weights["norm_final"])
            arrays = []
            for name in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_mlp"):
                arr = (C.c_void_p * m.n_layers)(*[dev(L[name]) for L in weights["layers"]])
                arrays.append(arr)
                setattr(w_c, name, C.cast(arr, C.POINTER(C.c_void_p)))
            cfg_p, w_p = C.byref(cfg_c), C.byref(w_c)
        rc = self._lib.ssd_create(C.byref(self._h), cfg_p, w_p, C.c_void_p(st.cuda_stream))
        if rc != 0:
            raise SsdError(rc, "ssd_create failed")

    def close(self):
        if self._h:
            self._lib.ssd_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc != 0:
            raise SsdError(rc, self._lib.ssd_last_error(self._h).decode())

    def workspace_bytes(self, max_frames=0, max_tokens=0, max_verify_rows=0, max_utts=0) -> int:
        return int(self._lib.ssd_workspace_bytes(self._h, max_frames, max_tokens, max_verify_rows, max_utts))

    def reserve(self, max_frames=0, max_tokens=0, max_verify_rows=0, max_utts=0, ar_utts=0, ar_steps=0):
        """Allocates (through torch) and hands over a workspace big enough for the given maxima."""
        n = self.workspace_bytes(max_frames, max_tokens, max_verify_rows, max_utts)
        if ar_utts and ar_steps:
            n = max(n, int(self._lib.ssd_ar_workspace_bytes(self._h, ar_utts, ar_steps)))
        if self._ws is None or self._ws.numel() < n:
            self._ws = torch.empty(n, dtype=torch.uint8, device=self.device)
            self._check(self._lib.ssd_set_workspace(self._h, _ptr(self._ws), n))

    def set_workspace(self, buf: Optional[torch.Tensor]):
        self._ws = buf
        self._check(self._lib.ssd_set_workspace(self._h, _ptr(buf), 0 if buf is None else buf.numel()))

    def inexact_weights(self) -> int:
        """Weight values whose conversion to the matrix-core operand type was not exact (0 for ordinary tensors)."""
        return int(self._lib.ssd_inexact_weights(self._h))

    def device_flags(self) -> int:
        """Sticky flags raised by kernels since the last call (waits for the stream); 1 = a token id was clamped,
        2 = an activation left the half range and was stored saturated (or a log-likelihood was not finite)."""
        f = C.c_int32(0)
        self._check(self._lib.ssd_device_flags(self._h, C.byref(f)))
        return int(f.value)

    def profile_select(self, kernel_class):
        k = PROF_CLASSES.index(kernel_class) if isinstance(kernel_class, str) else kernel_class
        self._check(self._lib.ssd_profile_select(self._h, k))

    def profile_read(self) -> dict:
        ms = np.zeros(len(PROF_CLASSES), dtype=np.float32)
        n = np.zeros(len(PROF_CLASSES), dtype=np.int32)
        self._check(self._lib.ssd_profile_read(self._h, ms.ctypes.data, n.ctypes.data))
        return {name: (float(ms[i]), int(n[i])) for i, name in enumerate(PROF_CLASSES)}

    def measure_mfma_ceiling(self, iters: int = 20000):
        t, g = C.c_float(), C.c_float()
        self._check(self._lib.ssd_measure_mfma_ceiling(self._h, iters, C.byref(t), C.byref(g)))
        return float(t.value), float(g.value)

    def measure_hbm_read(self, buf: torch.Tensor, iters: int = 5) -> float:
        g = C.c_float()
        self._check(self._lib.ssd_measure_hbm_read(self._h, buf.data_ptr(), buf.numel() * buf.element_size(), iters, C.byref(g)))
        return float(g.value)

    # ---- the three calls -------------------------------------------------------------------

    def ctc_gate(self, logits: torch.Tensor, cu_frames, blank_id: int, tau_ctc: float,
                 want_frames: bool = False, out: Optional[dict] = None) -> dict:
        cu = _host_i32(cu_frames)
        B, n_rows, V = len(cu) - 1, int(logits.shape[0]), int(logits.shape[1])
        dev = self.device
        if out is None:
            out = {"max_entropy": torch.empty(max(B, 0), dtype=torch.float32, device=dev),
                   "gate_pass": torch.empty(max(B, 0), dtype=torch.uint8, device=dev),
                   "draft_ctc": torch.empty(n_rows, dtype=torch.int32, device=dev),
                   "draft_len": torch.empty(max(B, 0), dtype=torch.int32, device=dev)}
            if want_frames:
                out["frame_entropy"] = torch.empty(n_rows, dtype=torch.float32, device=dev)
                out["frame_argmax"] = torch.empty(n_rows, dtype=torch.int32, device=dev)
        self._check(self._lib.ctc_gate(self._h, _ptr(logits), _DTYPE_CODE[logits.dtype], cu.ctypes.data, B, V,
                                       blank_id, tau_ctc, _ptr(out.get("frame_entropy")),
                                       _ptr(out.get("frame_argmax")), _ptr(out["max_entropy"]),
                                       _ptr(out["gate_pass"]), _ptr(out["draft_ctc"]), _ptr(out["draft_len"])))
        return out

    def set_ctc_head(self, w_ctc: torch.Tensor, bias: Optional[torch.Tensor] = None):
        """Output layer of the CTC encoder: w_ctc [V_ctc, d_enc] bf16, bias [V_ctc] fp32 (both on the device)."""
        if w_ctc.dtype != torch.bfloat16 or not w_ctc.is_contiguous():
            raise ValueError("w_ctc must be a contiguous bfloat16 tensor")
        if bias is not None and (bias.dtype != torch.float32 or bias.numel() != w_ctc.shape[0]):
            raise ValueError("bias must be float32 [V_ctc]")
        self._check(self._lib.ssd_set_ctc_head(self._h, _ptr(w_ctc), _ptr(bias), int(w_ctc.shape[0]), int(w_ctc.shape[1])))
        self._head_shape = (int(w_ctc.shape[0]), int(w_ctc.shape[1]))

    def ctc_head_gate(self, enc_h: torch.Tensor, cu_frames, blank_id: int, tau_ctc: float,
                      want_frames: bool = False) -> dict:
        cu = _host_i32(cu_frames)
        B, n_rows = len(cu) - 1, int(enc_h.shape[0])
        if enc_h.dtype != torch.bfloat16 or not enc_h.is_contiguous():
            raise ValueError("enc_h must be a contiguous bfloat16 tensor")
        shape = getattr(self, "_head_shape", None)
        if shape is not None and int(enc_h.shape[1]) != shape[1]:
            raise ValueError(f"enc_h has {enc_h.shape[1]} columns, the output layer expects {shape[1]}")
        dev = self.device
        out = {"max_entropy": torch.empty(max(B, 0), dtype=torch.float32, device=dev),
               "gate_pass": torch.empty(max(B, 0), dtype=torch.uint8, device=dev),
               "draft_ctc": torch.empty(n_rows, dtype=torch.int32, device=dev),
               "draft_len": torch.empty(max(B, 0), dtype=torch.int32, device=dev)}
        if want_frames:
            out["frame_entropy"] = torch.empty(n_rows, dtype=torch.float32, device=dev)
            out["frame_argmax"] = torch.empty(n_rows, dtype=torch.int32, device=dev)
        self._check(self._lib.ctc_head_gate(self._h, _ptr(enc_h), cu.ctypes.data, B, blank_id, tau_ctc,
                                            _ptr(out.get("frame_entropy")), _ptr(out.get("frame_argmax")),
                                            _ptr(out["max_entropy"]), _ptr(out["gate_pass"]),
                                            _ptr(out["draft_ctc"]), _ptr(out["draft_len"])))
        return out

    def select_unconfident(self, sel, cu_frames, draft_len_host, draft_ctc: torch.Tensor, ctc_to_llm: Optional[torch.Tensor],
                           speech_all: Optional[torch.Tensor], cu_speech_all, prompt_all: torch.Tensor, cu_prompt_all,
                           out: Optional[dict] = None, d_model: Optional[int] = None, dtype=None) -> dict:
        """ssd_select_unconfident: packed verification inputs of the utterances `sel` (host indices).  `out` may
        hold preallocated, large-enough `speech`, `prompt`, `draft_ids` tensors (their leading parts are written).
        speech_all may be None when cu_speech_all is all zero (no speech rows are moved); then d_model and dtype
        have to be given."""
        sel, cuf, dl = _host_i32(sel), _host_i32(cu_frames), _host_i32(draft_len_host)
        cs, cp = _host_i32(cu_speech_all), _host_i32(cu_prompt_all)
        n, B = len(sel), len(cuf) - 1
        d = int(speech_all.shape[1]) if speech_all is not None else int(d_model)
        sdt = speech_all.dtype if speech_all is not None else dtype
        nS = int((cs[sel + 1] - cs[sel]).sum()); nP = int((cp[sel + 1] - cp[sel]).sum()); nU = int(dl[sel].sum())
        if out is None:
            out = {"speech": torch.empty((nS, d), dtype=sdt, device=self.device),
                   "prompt": torch.empty(nP, dtype=torch.int32, device=self.device),
                   "draft_ids": torch.empty(nU, dtype=torch.int32, device=self.device)}
        assert out["speech"].shape[0] >= nS and out["prompt"].numel() >= nP and out["draft_ids"].numel() >= nU
        cso, cpo, cdo = (np.empty(n + 1, dtype=np.int32) for _ in range(3))
        V = 0 if ctc_to_llm is None else int(ctc_to_llm.numel())
        self._check(self._lib.ssd_select_unconfident(
            self._h, B, n, sel.ctypes.data, cuf.ctypes.data, dl.ctypes.data, _ptr(draft_ctc), _ptr(ctc_to_llm), V,
            _ptr(speech_all), cs.ctypes.data, _ptr(prompt_all), cp.ctypes.data, d, _DTYPE_CODE[sdt],
            _ptr(out["speech"]) if nS else None, _ptr(out["prompt"]) if nP else None, _ptr(out["draft_ids"]) if nU else None,
            cso.ctypes.data, cpo.ctypes.data, cdo.ctypes.data))
        return {"speech": out["speech"][:nS], "prompt": out["prompt"][:nP], "draft_ids": out["draft_ids"][:nU],
                "cu_speech": cso, "cu_prompt": cpo, "cu_draft": cdo}

    def gather_i32(self, src: torch.Tensor, idx, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """out[i] = src[idx[i]] on the device (ssd_gather_i32); idx is a host array."""
        ix = _host_i32(idx)
        if out is None:
            out = torch.empty(len(ix), dtype=torch.int32, device=self.device)
        self._check(self._lib.ssd_gather_i32(self._h, _ptr(src), ix.ctypes.data, len(ix), _ptr(out)))
        return out

    def set_qformer(self, q_proj: torch.Tensor, w_k: torch.Tensor, w_v: torch.Tensor, w_o: torch.Tensor, n_heads: int,
                    window: int = 15):
        """Projector windows (ssd_set_qformer): q_proj [n_q, d_h], w_k / w_v [d_h, d_enc], w_o [d_out, d_h], all bf16."""
        for t in (q_proj, w_k, w_v, w_o):
            if t.dtype != torch.bfloat16 or not t.is_contiguous():
                raise ValueError("projector weights must be contiguous bfloat16 tensors")
        n_q, d_h = int(q_proj.shape[0]), int(q_proj.shape[1])
        d_enc, d_out = int(w_k.shape[1]), int(w_o.shape[0])
        self._check(self._lib.ssd_set_qformer(self._h, _ptr(q_proj), _ptr(w_k), _ptr(w_v), _ptr(w_o), n_q, n_heads, d_h,
                                              d_enc, d_out, window))
        self._qformer = (n_q, d_enc, d_out, window)

    def qformer_pool(self, enc_h: torch.Tensor, cu_frames, out: Optional[torch.Tensor] = None):
        """Encoder frames -> acoustic embeddings (qformer_pool).  Returns (speech_emb [sum S, d_out] bf16, cu_speech)."""
        n_q, d_enc, d_out, window = self._qformer
        if enc_h.dtype != torch.bfloat16 or not enc_h.is_contiguous() or int(enc_h.shape[1]) != d_enc:
            raise ValueError("enc_h must be a contiguous bfloat16 tensor with d_enc columns")
        cu = _host_i32(cu_frames)
        B = len(cu) - 1
        n_rows = int(n_q * sum(-(-int(t) // window) for t in np.diff(cu)))
        if out is None:
            out = torch.empty((n_rows, d_out), dtype=torch.bfloat16, device=self.device)
        cu_s = np.empty(B + 1, dtype=np.int32)
        self._check(self._lib.qformer_pool(self._h, _ptr(enc_h), cu.ctypes.data, B, _ptr(out), cu_s.ctypes.data))
        return out[:n_rows], cu_s

    def verify_forward(self, speech_emb: torch.Tensor, cu_speech, prompt_ids: torch.Tensor, cu_prompt,
                       draft_ids: torch.Tensor, cu_draft, out: Optional[torch.Tensor] = None,
                       kv_start=None) -> torch.Tensor:
        """kv_start (host ints, one per utterance): also store keys/values in the K/V cache (verify_forward_kv)."""
        cs, cp, cd = _host_i32(cu_speech), _host_i32(cu_prompt), _host_i32(cu_draft)
        Bv = len(cd) - 1
        if out is None:
            out = torch.empty((int(cd[-1]), self.cfg.d_model), dtype=self.act_dtype, device=self.device)
        if kv_start is None:
            self._check(self._lib.verify_forward(self._h, _ptr(speech_emb), cs.ctypes.data, _ptr(prompt_ids),
                                                 cp.ctypes.data, _ptr(draft_ids), cd.ctypes.data, Bv, _ptr(out)))
        else:
            ks = _host_i32(kv_start)
            self._check(self._lib.verify_forward_kv(self._h, _ptr(speech_emb), cs.ctypes.data, _ptr(prompt_ids),
                                                    cp.ctypes.data, _ptr(draft_ids), cd.ctypes.data, Bv,
                                                    ks.ctypes.data, _ptr(out)))
        return out

    def gate_grid(self, max_entropy: torch.Tensor, taus_ctc) -> torch.Tensor:
        t = np.ascontiguousarray(np.asarray(taus_ctc, dtype=np.float32))
        B = int(max_entropy.numel())
        out = torch.empty((len(t), B), dtype=torch.uint8, device=self.device)
        self._check(self._lib.ssd_gate_grid(self._h, _ptr(max_entropy), B, t.ctypes.data, len(t), _ptr(out)))
        return out

    def accept_grid(self, draft_logp: torch.Tensor, cu_draft, taus_slm) -> dict:
        t = np.ascontiguousarray(np.asarray(taus_slm, dtype=np.float32))
        cd = _host_i32(cu_draft)
        Bv = len(cd) - 1
        out = {"accept_len": torch.empty((len(t), Bv), dtype=torch.int32, device=self.device),
               "all_accepted": torch.empty((len(t), Bv), dtype=torch.uint8, device=self.device)}
        self._check(self._lib.ssd_accept_grid(self._h, _ptr(draft_logp), cd.ctypes.data, Bv, t.ctypes.data, len(t),
                                              _ptr(out["accept_len"]), _ptr(out["all_accepted"])))
        return out

    def set_kv_cache(self, slots: int):
        """Allocates (through torch) a K/V cache of `slots` rows per layer and attaches it."""
        n = int(self._lib.ssd_kv_cache_bytes(self._h, slots))
        self._kv = torch.empty(n, dtype=torch.uint8, device=self.device)
        self._check(self._lib.ssd_set_kv_cache(self._h, _ptr(self._kv), n, slots))

    def ar_fallback(self, kv_start, ctx_len, first_tok: torch.Tensor, n_steps: int,
                    out: Optional[torch.Tensor] = None) -> torch.Tensor:
        ks, cl = _host_i32(kv_start), _host_i32(ctx_len)
        Br = len(ks)
        if out is None:
            out = torch.empty((n_steps, Br), dtype=torch.int32, device=self.device)
        self._check(self._lib.ar_fallback(self._h, Br, ks.ctypes.data, cl.ctypes.data, _ptr(first_tok), n_steps, _ptr(out)))
        return out

    def accept_prefix(self, h_verify: torch.Tensor, draft_ids: torch.Tensor, cu_draft, tau_slm: float,
                      want_greedy: bool = False, out: Optional[dict] = None) -> dict:
        cd = _host_i32(cu_draft)
        Bv, Mv = len(cd) - 1, int(cd[-1])
        dev = self.device
        if out is None:
            out = {"draft_logp": torch.empty(Mv, dtype=torch.float32, device=dev),
                   "accept_len": torch.empty(max(Bv, 0), dtype=torch.int32, device=dev),
                   "all_accepted": torch.empty(max(Bv, 0), dtype=torch.uint8, device=dev)}
            if want_greedy:
                out["greedy_tok"] = torch.empty(Mv, dtype=torch.int32, device=dev)
        self._check(self._lib.accept_prefix(self._h, _ptr(h_verify), _ptr(draft_ids), cd.ctypes.data, Bv, tau_slm,
                                            _ptr(out["draft_logp"]), _ptr(out["accept_len"]),
                                            _ptr(out["all_accepted"]), _ptr(out.get("greedy_tok"))))
        return out


NOALLOC_MAX_FRAMES = 262144


def ctc_gate_noalloc(logits: torch.Tensor, cu_frames_dev: torch.Tensor, blank_id: int, tau_ctc: float, out: dict,
                     stream=None) -> dict:
    """ctc_gate_noalloc: every buffer is the caller's (`out` holds max_entropy, gate_pass, draft_ctc, draft_len;
    cu_frames_dev is an int32 device tensor of B+1 prefix sums); the call itself allocates nothing."""
    st = stream if stream is not None else torch.cuda.current_stream(logits.device)
    B, n_frames, V = int(cu_frames_dev.numel()) - 1, int(logits.shape[0]), int(logits.shape[1])
    assert cu_frames_dev.dtype == torch.int32
    err = C.create_string_buffer(256)
    rc = lib().ctc_gate_noalloc(C.c_void_p(st.cuda_stream), _ptr(logits), _DTYPE_CODE[logits.dtype], _ptr(cu_frames_dev), B,
                                n_frames, V, blank_id, tau_ctc, _ptr(out["max_entropy"]), _ptr(out["gate_pass"]),
                                _ptr(out["draft_ctc"]), _ptr(out["draft_len"]), err, len(err))
    if rc != 0:
        raise SsdError(rc, err.value.decode())
    return out


def plan_batches(lengths, max_tokens: int, padded: bool = False):
    """Host-only batch planner (ssd_plan_batches): returns a list of index arrays, one per batch."""
    L = _host_i32(lengths)
    n = len(L)
    order = np.empty(n, dtype=np.int32)
    start = np.empty(n + 1, dtype=np.int32)
    nb = C.c_int32()
    rc = lib().ssd_plan_batches(L.ctypes.data, n, int(max_tokens), int(padded), order.ctypes.data, start.ctypes.data,
                                C.byref(nb))
    if rc != 0:
        raise SsdError(rc, "ssd_plan_batches: bad argument")
    return [order[start[k]:start[k + 1]].copy() for k in range(nb.value)]
