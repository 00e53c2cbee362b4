"""ctypes binding of libjdverify.so (argument marshalling only).

Function names mirror the C ABI in include/jd_verify.h.  Every step of the
verification path runs inside the HIP library; this module only hands over device
pointers taken from torch tensors.  There is no CPU fallback: if the shared library
is missing, importing the entry points raises.
"""

from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Dict, Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libjdverify.so")

JD_OK = 0
JD_ERR_INVALID_ARG, JD_ERR_SHAPE, JD_ERR_UNSUPPORTED_DTYPE, JD_ERR_OOM, JD_ERR_HIP = -1, -2, -3, -4, -5
JD_F32, JD_BF16, JD_FP8_E4M3, JD_INT8 = 0, 1, 2, 3
JD_W_VD, JD_W_DV = 0, 1
JD_DRAFT_LOGITS, JD_DRAFT_PROBS = 0, 1
JD_MODE_JUDGE, JD_MODE_STANDARD = 0, 1
JD_RULE_SAMPLING, JD_RULE_TOPK = 0, 1
JD_RESAMPLE_RESIDUAL, JD_RESAMPLE_TARGET = 0, 1
JD_STATUS_BAD_TOKEN, JD_STATUS_NAN, JD_STATUS_ZERO_RESIDUAL = 1, 2, 4
JD_K_LMHEAD, JD_K_DRAFTSTAT, JD_K_ACCEPT, JD_K_SAMPLER, JD_NUM_KERNELS = 0, 1, 2, 3, 4
KERNEL_NAMES = ("lmhead", "draftstat", "accept", "sampler")

EXPORTED_SYMBOLS = (
    "jd_verify_create", "jd_verify_create_scaled", "jd_verify_run", "jd_verify_run_prenorm", "jd_verify_append_tokens",
    "jd_verify_destroy", "jd_verify_strerror", "jd_verify_last_error_detail",
    "jd_verify_profile_begin", "jd_verify_profile_end", "jd_verify_workspace_bytes",
    "jd_verify_validate_config", "jd_verify_probe_mfma_bf16", "jd_verify_probe_hbm_read", "jd_verify_probe_hbm_read_plain",
    "jd_verify_run_noalloc",
)
JD_NOALLOC_SCRATCH_BYTES = 16 << 20


class jd_verify_config(ctypes.Structure):
    _fields_ = [
        ("d", ctypes.c_int32), ("V", ctypes.c_int32),
        ("max_B", ctypes.c_int32), ("max_M", ctypes.c_int32),
        ("w_dtype", ctypes.c_int32), ("emb_dtype", ctypes.c_int32),
        ("w_layout", ctypes.c_int32), ("draft_kind", ctypes.c_int32), ("mode", ctypes.c_int32),
        ("temperature", ctypes.c_float), ("delta", ctypes.c_float), ("judge_bias", ctypes.c_float),
        ("device", ctypes.c_int32),
        ("rule", ctypes.c_int32), ("top_k", ctypes.c_int32), ("resample", ctypes.c_int32),
    ]


class jd_verify_outputs(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in (
        "d_accept_len", "d_next_token", "d_status", "d_z_stand", "d_z_judge", "d_p_at_draft",
        "d_q_at_draft", "d_judge_logit", "d_row_max", "d_row_sumexp", "d_probs")]


class JDError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        detail = ""
        if code in (JD_ERR_HIP, JD_ERR_OOM) and _lib is not None:
            detail = (_lib.jd_verify_last_error_detail() or b"").decode()
        super().__init__(f"{where}: {strerror(code)} ({code})" + (f" [{detail}]" if detail else ""))


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libjdverify.so; fail loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2501_19309_amd.build` "
            "(there is no fallback path)")
    # The device tensors this binding hands over come from PyTorch, which ships its own copy of the HIP
    # runtime.  Loading PyTorch first makes the library's libamdhip64 dependency resolve to that same,
    # already loaded copy; the other order puts two runtimes into the process and the second one finds
    # no device ("no ROCm-capable device is detected" from every call of the library).
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32 = ctypes.c_void_p, ctypes.c_int32
    lib.jd_verify_create.argtypes = [ctypes.POINTER(jd_verify_config), vp, vp, ctypes.POINTER(vp)]
    lib.jd_verify_create.restype = ctypes.c_int
    lib.jd_verify_create_scaled.argtypes = [ctypes.POINTER(jd_verify_config), vp, vp, vp, ctypes.POINTER(vp)]
    lib.jd_verify_create_scaled.restype = ctypes.c_int
    lib.jd_verify_run.argtypes = [vp, i32, i32, vp, vp, vp, vp, i32, vp, ctypes.POINTER(jd_verify_outputs), vp]
    lib.jd_verify_run.restype = ctypes.c_int
    lib.jd_verify_run_prenorm.argtypes = [vp, i32, i32, vp, vp, ctypes.c_double, vp, vp, i32, vp,
                                          ctypes.POINTER(jd_verify_outputs), vp]
    lib.jd_verify_run_prenorm.restype = ctypes.c_int
    lib.jd_verify_run_noalloc.argtypes = [ctypes.POINTER(jd_verify_config), vp, vp, i32, i32, vp, vp, vp, vp, i32, vp,
                                          ctypes.POINTER(jd_verify_outputs), vp]
    lib.jd_verify_run_noalloc.restype = ctypes.c_int
    lib.jd_verify_append_tokens.argtypes = [i32, i32, vp, vp, vp, vp, i32, vp, vp]
    lib.jd_verify_append_tokens.restype = ctypes.c_int
    lib.jd_verify_destroy.argtypes = [vp]
    lib.jd_verify_destroy.restype = ctypes.c_int
    lib.jd_verify_strerror.argtypes = [ctypes.c_int]
    lib.jd_verify_strerror.restype = ctypes.c_char_p
    lib.jd_verify_last_error_detail.argtypes = []
    lib.jd_verify_last_error_detail.restype = ctypes.c_char_p
    lib.jd_verify_profile_begin.argtypes = [vp, i32]
    lib.jd_verify_profile_begin.restype = ctypes.c_int
    lib.jd_verify_profile_end.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32)]
    lib.jd_verify_profile_end.restype = ctypes.c_int
    lib.jd_verify_workspace_bytes.argtypes = [vp, ctypes.POINTER(ctypes.c_uint64)]
    lib.jd_verify_workspace_bytes.restype = ctypes.c_int
    lib.jd_verify_validate_config.argtypes = [ctypes.POINTER(jd_verify_config)]
    lib.jd_verify_validate_config.restype = ctypes.c_int
    lib.jd_verify_probe_mfma_bf16.argtypes = [i32, i32, ctypes.POINTER(ctypes.c_double)]
    lib.jd_verify_probe_mfma_bf16.restype = ctypes.c_int
    lib.jd_verify_probe_hbm_read.argtypes = [i32, ctypes.c_uint64, ctypes.POINTER(ctypes.c_double)]
    lib.jd_verify_probe_hbm_read.restype = ctypes.c_int
    lib.jd_verify_probe_hbm_read_plain.argtypes = [i32, ctypes.c_uint64, ctypes.POINTER(ctypes.c_double)]
    lib.jd_verify_probe_hbm_read_plain.restype = ctypes.c_int
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load_library().jd_verify_strerror(int(code)).decode()


def make_config(d, V, max_B, max_M, *, w_dtype=JD_BF16, emb_dtype=None, w_layout=JD_W_VD,
                draft_kind=JD_DRAFT_LOGITS, mode=JD_MODE_JUDGE, temperature=1.0, delta=0.5,
                judge_bias=0.0, device=0, rule=JD_RULE_SAMPLING, top_k=1,
                resample=JD_RESAMPLE_RESIDUAL) -> jd_verify_config:
    if emb_dtype is None:
        emb_dtype = JD_BF16 if w_dtype in (JD_FP8_E4M3, JD_INT8) else w_dtype
    return jd_verify_config(d, V, max_B, max_M, w_dtype, emb_dtype,
                            w_layout, draft_kind, mode, temperature, delta, judge_bias, device,
                            rule, top_k, resample)


def jd_verify_validate_config(cfg: jd_verify_config) -> int:
    return load_library().jd_verify_validate_config(ctypes.byref(cfg))


def probe_mfma_bf16(device: int = 0, operand_mode: int = 1) -> float:
    """jd_verify_probe_mfma_bf16: TFLOP/s of a loop of nothing but independent bf16 MFMAs on this device."""
    v = ctypes.c_double()
    rc = load_library().jd_verify_probe_mfma_bf16(device, operand_mode, ctypes.byref(v))
    if rc != JD_OK:
        raise JDError(rc, "jd_verify_probe_mfma_bf16")
    return float(v.value)


def probe_hbm_read(device: int = 0, nbytes: int = 4 << 30, plain_loads: bool = False) -> float:
    """jd_verify_probe_hbm_read(_plain): GB/s of a pure streaming read of an nbytes buffer on this device, with
    non-temporal loads (as the library streams its weights) or, for the comparison, with plain ones."""
    v = ctypes.c_double()
    name = "jd_verify_probe_hbm_read_plain" if plain_loads else "jd_verify_probe_hbm_read"
    rc = getattr(load_library(), name)(device, nbytes, ctypes.byref(v))
    if rc != JD_OK:
        raise JDError(rc, name)
    return float(v.value)


def append_tokens(draft_tokens, accept_len, next_token, token_buf, lengths, stream=None) -> None:
    """jd_verify_append_tokens on torch device tensors (int32): grows token_buf [B, cap] / lengths [B] in place."""
    import torch
    B, M = draft_tokens.shape
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    rc = load_library().jd_verify_append_tokens(B, M, _ptr(draft_tokens), _ptr(accept_len), _ptr(next_token),
                                                _ptr(token_buf), token_buf.shape[1], _ptr(lengths),
                                                ctypes.c_void_p(stream))
    if rc != JD_OK:
        raise JDError(rc, "jd_verify_append_tokens")


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def alloc_outputs(B: int, M: int, V: int = 0, want_probs: bool = False, device: int = 0) -> "VerifyOutputs":
    """Device tensors for the outputs of one verify call."""
    import torch as t
    dev = t.device("cuda", device)
    f = lambda *s: t.zeros(*s, dtype=t.float32, device=dev)
    return VerifyOutputs(
        accept_len=t.zeros(B, dtype=t.int32, device=dev), next_token=t.zeros(B, dtype=t.int32, device=dev),
        status=t.zeros(B, dtype=t.int32, device=dev),
        z_stand=t.zeros(B, M, dtype=t.uint8, device=dev), z_judge=t.zeros(B, M, dtype=t.uint8, device=dev),
        p_at_draft=f(B, M), q_at_draft=f(B, M), judge_logit=f(B, M), row_max=f(B, M + 1),
        row_sumexp=f(B, M + 1), probs=f(B, M + 1, V) if want_probs else None)


def outputs_struct(out: "VerifyOutputs") -> jd_verify_outputs:
    return jd_verify_outputs(*[_ptr(getattr(out, n)) for n in (
        "accept_len", "next_token", "status", "z_stand", "z_judge", "p_at_draft", "q_at_draft",
        "judge_logit", "row_max", "row_sumexp", "probs")])


def run_noalloc_raw(cfg: jd_verify_config, W_lm, w_judge, B, M, emb, emb_judge, draft_tokens, draft, draft_rows,
                    uniforms, outputs: Optional[jd_verify_outputs], stream=0) -> int:
    """jd_verify_run_noalloc with raw device pointers (ints or None); returns the error code."""
    return load_library().jd_verify_run_noalloc(ctypes.byref(cfg), W_lm, w_judge, B, M, emb, emb_judge, draft_tokens,
                                                draft, draft_rows, uniforms,
                                                ctypes.byref(outputs) if outputs is not None else None,
                                                ctypes.c_void_p(stream))


def run_noalloc(cfg: jd_verify_config, W_lm, w_judge, emb, draft_tokens, draft, uniforms, out: "VerifyOutputs", *,
                emb_judge=None, stream=None) -> None:
    """jd_verify_run_noalloc on torch device tensors: one verify call without a context (fp32 weights), the
    workspace in the library's static device array."""
    import torch
    B, M = emb.shape[0], emb.shape[1] - 1
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    rc = run_noalloc_raw(cfg, _ptr(W_lm), _ptr(w_judge), B, M, _ptr(emb), _ptr(emb_judge), _ptr(draft_tokens),
                         _ptr(draft), draft.shape[1], _ptr(uniforms), outputs_struct(out), stream)
    if rc != JD_OK:
        raise JDError(rc, "jd_verify_run_noalloc")


@dataclass
class VerifyOutputs:
    """Device tensors written by one jd_verify_run call."""
    accept_len: "torch.Tensor"
    next_token: "torch.Tensor"
    status: "torch.Tensor"
    z_stand: "torch.Tensor"
    z_judge: "torch.Tensor"
    p_at_draft: "torch.Tensor"
    q_at_draft: "torch.Tensor"
    judge_logit: "torch.Tensor"
    row_max: "torch.Tensor"
    row_sumexp: "torch.Tensor"
    probs: Optional["torch.Tensor"] = None

    def to_numpy(self) -> Dict[str, "numpy.ndarray"]:
        out = {}
        for k, v in self.__dict__.items():
            if v is not None:
                out[k] = v.detach().cpu().numpy()
        return out


class JDVerify:
    """Owner of one jd_verify_ctx.  Tensors are torch CUDA(HIP) tensors."""

    def __init__(self, cfg: jd_verify_config, W_lm, w_judge, w_scale=None):
        import torch  # device memory and streams only

        self._torch = torch
        self.lib = load_library()
        self.cfg = cfg
        self._keep = (W_lm, w_judge, w_scale)  # borrowed by the library until destroy
        handle = ctypes.c_void_p()
        if w_scale is None:
            rc = self.lib.jd_verify_create(ctypes.byref(cfg), _ptr(W_lm), _ptr(w_judge), ctypes.byref(handle))
        else:
            rc = self.lib.jd_verify_create_scaled(ctypes.byref(cfg), _ptr(W_lm), _ptr(w_scale), _ptr(w_judge),
                                                  ctypes.byref(handle))
        if rc != JD_OK:
            raise JDError(rc, "jd_verify_create")
        self.handle = handle

    # -- jd_verify_run
    def alloc_outputs(self, B: int, M: int, want_probs: bool = False) -> VerifyOutputs:
        return alloc_outputs(B, M, self.cfg.V, want_probs, self.cfg.device)

    def run(self, emb, draft_tokens, draft, uniforms, out: VerifyOutputs, *, emb_judge=None, stream=None) -> None:
        B, Mp1 = emb.shape[0], emb.shape[1]
        M = Mp1 - 1
        o = jd_verify_outputs(*[_ptr(getattr(out, n)) for n in (
            "accept_len", "next_token", "status", "z_stand", "z_judge", "p_at_draft", "q_at_draft",
            "judge_logit", "row_max", "row_sumexp", "probs")])
        if stream is None:
            stream = self._torch.cuda.current_stream().cuda_stream
        rc = self.lib.jd_verify_run(self.handle, B, M, _ptr(emb), _ptr(emb_judge), _ptr(draft_tokens), _ptr(draft),
                                    draft.shape[1], _ptr(uniforms), ctypes.byref(o), ctypes.c_void_p(stream))
        if rc != JD_OK:
            raise JDError(rc, "jd_verify_run")

    def run_prenorm(self, hidden, gamma, rms_eps: float, draft_tokens, draft, uniforms, out: VerifyOutputs, *,
                    stream=None) -> None:
        """jd_verify_run_prenorm: pre-norm hidden states in, normalised for the LM head by the library."""
        B, Mp1 = hidden.shape[0], hidden.shape[1]
        M = Mp1 - 1
        o = jd_verify_outputs(*[_ptr(getattr(out, n)) for n in (
            "accept_len", "next_token", "status", "z_stand", "z_judge", "p_at_draft", "q_at_draft",
            "judge_logit", "row_max", "row_sumexp", "probs")])
        if stream is None:
            stream = self._torch.cuda.current_stream().cuda_stream
        rc = self.lib.jd_verify_run_prenorm(self.handle, B, M, _ptr(hidden), _ptr(gamma), float(rms_eps),
                                            _ptr(draft_tokens), _ptr(draft), draft.shape[1], _ptr(uniforms),
                                            ctypes.byref(o), ctypes.c_void_p(stream))
        if rc != JD_OK:
            raise JDError(rc, "jd_verify_run_prenorm")

    def run_prenorm_raw(self, B, M, hidden, gamma, rms_eps, draft_tokens, draft, draft_rows, uniforms,
                        outputs: jd_verify_outputs, stream=0) -> int:
        """Direct call returning the error code (used by the error-path tests)."""
        return self.lib.jd_verify_run_prenorm(self.handle, B, M, hidden, gamma, float(rms_eps), draft_tokens, draft,
                                              draft_rows, uniforms,
                                              ctypes.byref(outputs) if outputs is not None else None,
                                              ctypes.c_void_p(stream))

    def run_raw(self, B, M, emb, emb_judge, draft_tokens, draft, draft_rows, uniforms, outputs: jd_verify_outputs,
                stream=0) -> int:
        """Direct call returning the error code (used by the error-path tests)."""
        return self.lib.jd_verify_run(self.handle, B, M, emb, emb_judge, draft_tokens, draft, draft_rows, uniforms,
                                      ctypes.byref(outputs) if outputs is not None else None, ctypes.c_void_p(stream))

    # -- profiling
    def profile_begin(self, max_calls: int) -> None:
        rc = self.lib.jd_verify_profile_begin(self.handle, max_calls)
        if rc != JD_OK:
            raise JDError(rc, "jd_verify_profile_begin")

    def profile_end(self):
        ms = (ctypes.c_float * JD_NUM_KERNELS)()
        n = ctypes.c_int32()
        rc = self.lib.jd_verify_profile_end(self.handle, ms, ctypes.byref(n))
        if rc != JD_OK:
            raise JDError(rc, "jd_verify_profile_end")
        return {KERNEL_NAMES[i]: float(ms[i]) for i in range(JD_NUM_KERNELS)}, int(n.value)

    def workspace_bytes(self) -> int:
        v = ctypes.c_uint64()
        rc = self.lib.jd_verify_workspace_bytes(self.handle, ctypes.byref(v))
        if rc != JD_OK:
            raise JDError(rc, "jd_verify_workspace_bytes")
        return int(v.value)

    # -- jd_verify_destroy
    def destroy(self) -> None:
        if getattr(self, "handle", None) is not None:
            self.lib.jd_verify_destroy(self.handle)
            self.handle = None
            self._keep = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
