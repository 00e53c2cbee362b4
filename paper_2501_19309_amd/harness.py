"""Host-side plumbing shared by the GPU tests, the smoke check and the benchmark:
moves numpy input dicts (as produced by ``synth.make_inputs``) into device memory and
drives the C-ABI library.  No verification arithmetic happens here.
"""

from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from . import binding as jb


def to_device(inputs: Dict[str, np.ndarray], device: int = 0):
    """numpy -> torch device tensors; uint16 arrays are bf16 bit patterns, uint8 arrays FP8 codes, int8 arrays INT8 weights."""
    import torch

    dev = torch.device("cuda", device)
    out = {}
    for k in ("emb", "hidden", "gamma", "W", "w_judge", "w_scale", "draft_logits", "draft_tokens", "uniforms",
              "emb_judge", "draft_probs"):
        if k not in inputs or inputs[k] is None:
            continue
        a = np.ascontiguousarray(inputs[k])
        if a.dtype == np.uint16:
            t = torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        else:
            t = torch.from_numpy(a).to(dev)
        out[k] = t
    return out


def make_verifier(dev_inputs, *, max_B: Optional[int] = None, max_M: Optional[int] = None, device: int = 0,
                  w_layout: int = jb.JD_W_VD, **cfg_kw) -> jb.JDVerify:
    import torch

    emb, W = dev_inputs.get("emb", dev_inputs.get("hidden")), dev_inputs["W"]
    B, Mp1, d = emb.shape
    V = W.shape[0] if w_layout == jb.JD_W_VD else W.shape[1]
    dt = {torch.bfloat16: jb.JD_BF16, torch.uint8: jb.JD_FP8_E4M3, torch.int8: jb.JD_INT8}.get(W.dtype, jb.JD_F32)
    cfg = jb.make_config(d, V, max_B or B, max_M or (Mp1 - 1), w_dtype=dt, w_layout=w_layout, device=device,
                         **cfg_kw)
    return jb.JDVerify(cfg, W, dev_inputs["w_judge"], dev_inputs.get("w_scale"))


def run_once(inputs: Dict[str, np.ndarray], *, want_probs: bool = False, device: int = 0,
             w_layout: int = jb.JD_W_VD, **cfg_kw) -> Dict[str, np.ndarray]:
    """Upload, create a context, run one verify call, download every output."""
    import torch

    dev_in = to_device(inputs, device)
    ver = make_verifier(dev_in, device=device, w_layout=w_layout, **cfg_kw)
    try:
        emb = dev_in.get("emb", dev_in.get("hidden"))
        B, M = emb.shape[0], emb.shape[1] - 1
        out = ver.alloc_outputs(B, M, want_probs)
        draft = dev_in["draft_probs"] if cfg_kw.get("draft_kind", jb.JD_DRAFT_LOGITS) == jb.JD_DRAFT_PROBS \
            else dev_in["draft_logits"]
        if "hidden" in dev_in:   # pre-norm wiring: the library normalises, the judge reads the hidden states
            ver.run_prenorm(dev_in["hidden"], dev_in["gamma"], float(inputs["rms_eps"]), dev_in["draft_tokens"], draft,
                            dev_in["uniforms"], out)
        else:
            ver.run(emb, dev_in["draft_tokens"], draft, dev_in["uniforms"], out, emb_judge=dev_in.get("emb_judge"))
        torch.cuda.synchronize(device)
        return out.to_numpy()
    finally:
        ver.destroy()
