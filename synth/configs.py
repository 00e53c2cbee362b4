"""Seeded synthetic workloads shaped like the paper's Llama-3.1 target models.

The paper evaluates Llama-3.1-8B drafting for Llama-3.1-70B / 405B targets
(Sec. 5, Table 1; judge width 8192 / 16384 in App. B.1; M = 25 judge drafts and
M = 10 standard drafts in Sec. 5; 8-bit target weights in Table 1 and App. B.3).  None of those weights or prompts exist here,
so these generators stand in for them: same shapes, Gaussian statistics chosen so
that logits have unit variance and the draft is a noisy copy of the target.

Every array is a pure function of ``(shape, seed)``.  Randomness comes from
numpy's counter-based Philox generator, one independent stream per (tensor tag,
vocabulary chunk), so chunks can be drawn in parallel threads and the result does
not depend on the thread count.

Nothing in this file is part of the verification method: the only arithmetic is
drawing numbers, rounding to bf16 (or quantising the drawn weights to FP8 E4M3 with
one scale per row), one single-precision matmul to make the draft logits a perturbed
copy of the target logits (for the pre-norm workloads preceded by a single-precision
normalisation of the drawn hidden states, used for nothing else: the oracle and the
library each normalise the stored hidden states themselves), and a Gumbel arg-max to
draw the draft tokens from the draft distribution.
"""

from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Dict, Optional, Tuple, Union

import numpy as np

# tensor tags: each selects its own family of Philox streams
_TAG_EMB, _TAG_W, _TAG_JUDGE, _TAG_SCALE, _TAG_NOISE, _TAG_GUMBEL, _TAG_UNIF, _TAG_GAMMA, _TAG_ROWSCALE = range(1, 10)

RMS_EPS = 1e-5  # epsilon of the final RMS normalisation in the pre-norm workloads

_VOCAB_CHUNK = 2048  # rows of W_lm drawn per Philox stream


@dataclass(frozen=True)
class VerifyShape:
    """One verification workload: B sequences, M drafted tokens (+1 bonus row)."""

    name: str
    B: int
    M: int
    d: int
    V: int
    dtype: str  # "f32" | "bf16": storage type of embeddings, W_lm and w_judge;
                # "fp8": bf16 embeddings and w_judge, W_lm as FP8 E4M3 codes + one fp32 scale per row
                # "int8": the same with W_lm as two's-complement 8-bit integers
    noise: Union[float, Tuple[float, float]]  # std of draft-logit noise, or U(lo, hi) per sequence
    note: str = ""

    @property
    def R(self) -> int:
        return self.B * (self.M + 1)


CONFIGS: Dict[str, VerifyShape] = {
    "C1": VerifyShape("C1", 1, 5, 256, 1024, "f32", 1.0, "tiny oracle-scale verify, fp32"),
    "C2": VerifyShape("C2", 1, 5, 4096, 128256, "bf16", 1.5, "Llama-3.1-8B-shaped head"),
    "C3": VerifyShape("C3", 1, 25, 8192, 128256, "bf16", 1.0, "Llama-3.1-70B-shaped head, long drafts"),
    "C4": VerifyShape("C4", 1, 25, 16384, 128256, "bf16", 2.0, "Llama-3.1-405B-shaped head (headline, HBM bound)"),
    "C5": VerifyShape("C5", 64, 10, 8192, 128256, "bf16", (0.5, 2.5), "batched verification (MFMA bound)"),
    # 8-bit weight variants (the paper's runs quantise the target to 8 bits): same shapes, FP8 E4M3 W_lm
    "C2q": VerifyShape("C2q", 1, 5, 4096, 128256, "fp8", 1.5, "Llama-3.1-8B-shaped head, FP8 W_lm"),
    "C3q": VerifyShape("C3q", 1, 25, 8192, 128256, "fp8", 1.0, "Llama-3.1-70B-shaped head, FP8 W_lm"),
    "C4q": VerifyShape("C4q", 1, 25, 16384, 128256, "fp8", 2.0, "Llama-3.1-405B-shaped head, FP8 W_lm"),
    "C5q": VerifyShape("C5q", 64, 10, 8192, 128256, "fp8", (0.5, 2.5), "batched verification, FP8 W_lm"),
    # the same with 8-bit integer weights and one scale per output channel (weight-only quantisation)
    "C2i": VerifyShape("C2i", 1, 5, 4096, 128256, "int8", 1.5, "Llama-3.1-8B-shaped head, INT8 W_lm"),
    "C3i": VerifyShape("C3i", 1, 25, 8192, 128256, "int8", 1.0, "Llama-3.1-70B-shaped head, INT8 W_lm"),
    "C4i": VerifyShape("C4i", 1, 25, 16384, 128256, "int8", 2.0, "Llama-3.1-405B-shaped head, INT8 W_lm"),
    "C5i": VerifyShape("C5i", 64, 10, 8192, 128256, "int8", (0.5, 2.5), "batched verification, INT8 W_lm"),
}


def bf16_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def f32_from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _e4m3fn_positive_values() -> np.ndarray:
    """The 127 finite non-negative FP8 E4M3 ("fn") values, code order (code = index)."""
    vals = []
    for code in range(127):
        e, m = (code >> 3) & 0xF, code & 0x7
        vals.append(m * 2.0 ** -9 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7))
    return np.asarray(vals, dtype=np.float32)


_E4M3_POS = _e4m3fn_positive_values()
_E4M3_MID = ((_E4M3_POS[:-1].astype(np.float64) + _E4M3_POS[1:].astype(np.float64)) / 2).astype(np.float32)


def fp8_e4m3_quantize_rows(w: np.ndarray):
    """Per-row symmetric quantisation of float32 rows to FP8 E4M3 codes.

    scale[v] = max|w[v,:]| / 448 (float32); code = nearest representable value of w / scale.
    Returns (codes uint8 [rows, d], scale float32 [rows], dequantised float32 [rows, d]).
    """
    amax = np.max(np.abs(w), axis=1).astype(np.float32)
    scale = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    q = w / scale[:, None]
    mag = np.searchsorted(_E4M3_MID, np.abs(q)).astype(np.uint8)      # nearest code of |q| (0..126)
    codes = mag | (np.signbit(q).astype(np.uint8) << 7)
    deq = _E4M3_POS[mag] * np.where(np.signbit(q), np.float32(-1), np.float32(1)) * scale[:, None]
    return codes, scale, deq.astype(np.float32)


def int8_quantize_rows(w: np.ndarray):
    """Per-row symmetric weight-only quantisation of float32 rows to 8-bit integers (one scale per
    output channel, the usual recipe of 8-bit weight-only inference).

    scale[v] = max|w[v,:]| / 127 (float32); code = round-half-even(w / scale) in [-127, 127].
    Returns (codes int8 [rows, d], scale float32 [rows], dequantised float32 [rows, d]).
    """
    amax = np.max(np.abs(w), axis=1).astype(np.float32)
    scale = np.where(amax > 0, amax / np.float32(127.0), np.float32(1.0)).astype(np.float32)
    q = np.clip(np.rint(w / scale[:, None]), -127, 127)
    codes = q.astype(np.int8)
    return codes, scale, (q.astype(np.float32) * scale[:, None]).astype(np.float32)


def _stream(seed: int, tag: int, chunk: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64((tag << 40) | chunk)]))


def _n_threads() -> int:
    try:
        avail = len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        avail = os.cpu_count() or 1
    return max(1, min(16, avail))


def make_inputs(shape: VerifyShape, seed: int = 0, prenorm: bool = False,
                weights_seed: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Draw every input of one verify call.

    weights_seed (default: seed) selects the streams of the model's own tensors (W_lm, w_judge, the
    norm gain): several calls with one weights_seed and different seeds are different batches for the
    same model, as a decode loop sees them.

    prenorm=True draws the workload in the paper's wiring (Sec. 4.1: the judge sees the last target
    embedding before the final RMS normalisation): instead of ``emb`` the dict holds
      hidden        [B, M+1, d]  pre-norm hidden states (rows of very different scale), storage type
      gamma         [d]          gain of the final RMS normalisation, storage type
      rms_eps       float
    and the draft logits are a noisy copy of the logits of a single-precision normalisation of them.

    Returns a dict with
      emb           [B, M+1, d]  float32, or uint16 bf16 bit patterns
      W             [V, d]       same storage type; row v is vocabulary entry v (K contiguous);
                                 for dtype "fp8": uint8 FP8 E4M3 codes, plus  w_scale [V] float32;
                                 for dtype "int8": int8 weights, plus  w_scale [V] float32
      w_judge       [d]          same storage type
      draft_logits  [B, M+1, V]  float32 (row M is present but unused by verification)
      draft_tokens  [B, M]       int32, token j drawn from softmax(draft_logits[:, j])
      uniforms      [B, M+1]     float32 in [0, 1): M accept draws, then one sampler draw
    """
    B, M, d, V = shape.B, shape.M, shape.d, shape.V
    R = B * (M + 1)
    is_fp8, is_int8 = shape.dtype == "fp8", shape.dtype == "int8"
    is_w8 = is_fp8 or is_int8
    is_bf16 = shape.dtype == "bf16" or is_w8   # storage of embeddings and w_judge
    if shape.dtype not in ("f32", "bf16", "fp8", "int8"):
        raise ValueError(f"unknown dtype {shape.dtype!r}")

    # embeddings: N(0,1), each row rescaled to unit rms, then stored
    h = _stream(seed, _TAG_EMB).standard_normal((R, d), dtype=np.float32)
    h /= np.sqrt(np.mean(h.astype(np.float64) ** 2, axis=1, keepdims=True)).astype(np.float32)
    hidden_store = gamma_store = None
    if prenorm:
        # pre-norm hidden states: the unit-rms rows times a log-normal scale per row; gain near 1
        rowscale = np.exp(_stream(seed, _TAG_ROWSCALE).standard_normal(R).astype(np.float32) * np.float32(0.7))
        hid = h * rowscale[:, None] * np.float32(3.0)
        gam = (np.float32(1.0) + np.float32(0.1) * _stream(seed if weights_seed is None else weights_seed, _TAG_GAMMA).standard_normal(d, dtype=np.float32))
        if is_bf16:
            hidden_store = bf16_bits_from_f32(hid); hid = f32_from_bf16_bits(hidden_store)
            gamma_store = bf16_bits_from_f32(gam); gam = f32_from_bf16_bits(gamma_store)
        else:
            hidden_store, gamma_store = hid.copy(), gam.copy()
        # a single-precision stand-in for the LM-head input, only used to build the draft logits below
        h = hid * gam / np.sqrt(np.mean(hid.astype(np.float64) ** 2, axis=1, keepdims=True) + RMS_EPS).astype(np.float32)
    if is_bf16:
        emb_store = bf16_bits_from_f32(h)
        h = f32_from_bf16_bits(emb_store)
    else:
        emb_store = h.copy()

    wseed = seed if weights_seed is None else weights_seed
    wj = _stream(wseed, _TAG_JUDGE).standard_normal(d, dtype=np.float32) * np.float32(1.0 / np.sqrt(d))
    wj_store = bf16_bits_from_f32(wj) if is_bf16 else wj

    if isinstance(shape.noise, tuple):
        lo, hi = shape.noise
        sigma_b = _stream(seed, _TAG_SCALE).uniform(lo, hi, size=B).astype(np.float32)
    else:
        sigma_b = np.full(B, shape.noise, dtype=np.float32)
    sigma_r = np.repeat(sigma_b, M + 1)[:, None]  # [R, 1]

    W_store = np.empty((V, d), dtype=np.uint8 if is_fp8 else np.int8 if is_int8 else (np.uint16 if is_bf16 else np.float32))
    W_scale = np.ones(V, dtype=np.float32)
    D = np.empty((R, V), dtype=np.float32)
    best_val = np.full(R, -np.inf, dtype=np.float32)
    best_idx = np.zeros(R, dtype=np.int64)
    inv_sqrt_d = np.float32(1.0 / np.sqrt(d))

    def draw_chunk(ci: int):
        v0 = ci * _VOCAB_CHUNK
        rows = min(_VOCAB_CHUNK, V - v0)
        w = _stream(wseed, _TAG_W, ci).standard_normal((rows, d), dtype=np.float32)
        w *= inv_sqrt_d
        noise = _stream(seed, _TAG_NOISE, ci).standard_normal((R, rows), dtype=np.float32)
        gumbel = _stream(seed, _TAG_GUMBEL, ci).gumbel(size=(R, rows)).astype(np.float32)
        if is_w8:
            codes, scale, deq = fp8_e4m3_quantize_rows(w) if is_fp8 else int8_quantize_rows(w)
            return ci, codes, noise, gumbel, scale, deq
        w_bits = bf16_bits_from_f32(w) if is_bf16 else None
        return ci, (w_bits if is_bf16 else w), noise, gumbel, None, None

    n_chunks = (V + _VOCAB_CHUNK - 1) // _VOCAB_CHUNK
    nthreads = _n_threads()
    with ThreadPoolExecutor(max_workers=nthreads) as pool:
        # keep at most ~2*nthreads chunks in flight so float32 temporaries stay bounded
        pending = []
        next_ci = 0

        def top_up():
            nonlocal next_ci
            while next_ci < n_chunks and len(pending) < 2 * nthreads:
                pending.append(pool.submit(draw_chunk, next_ci))
                next_ci += 1

        top_up()
        while pending:
            ci, w_chunk, noise, gumbel, scale, deq = pending.pop(0).result()
            top_up()
            v0 = ci * _VOCAB_CHUNK
            rows = w_chunk.shape[0]
            W_store[v0:v0 + rows] = w_chunk
            if is_w8:
                W_scale[v0:v0 + rows] = scale
                w32 = deq
            else:
                w32 = f32_from_bf16_bits(w_chunk) if is_bf16 else w_chunk
            # draft logits = (single-precision) target logits + Gaussian noise
            Dc = h @ w32.T
            Dc += sigma_r * noise
            D[:, v0:v0 + rows] = Dc
            # Gumbel arg-max draws one token per row from softmax(D[row])
            g = Dc + gumbel
            loc = np.argmax(g, axis=1)
            val = g[np.arange(R), loc]
            upd = val > best_val
            best_val[upd] = val[upd]
            best_idx[upd] = loc[upd] + v0

    tokens = best_idx.reshape(B, M + 1)[:, :M].astype(np.int32)
    uniforms = _stream(seed, _TAG_UNIF).random((B, M + 1), dtype=np.float32)

    out = {
        "W": W_store,
        "w_judge": wj_store,
        "draft_logits": D.reshape(B, M + 1, V),
        "draft_tokens": np.ascontiguousarray(tokens),
        "uniforms": uniforms,
        "sigma_b": sigma_b,
    }
    if prenorm:
        out["hidden"] = hidden_store.reshape(B, M + 1, d)
        out["gamma"] = gamma_store
        out["rms_eps"] = RMS_EPS
    else:
        out["emb"] = emb_store.reshape(B, M + 1, d)
    if is_w8:
        out["w_scale"] = W_scale
    return out
