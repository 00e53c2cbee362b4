"""Float64 CPU oracle for the Judge-Decoding verification head.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the HIP
library is checked against.  It shares no code with the HIP path and must never
be imported by it; only the tests, the smoke check and the benchmark's
``cpu_baseline`` leg call it.

What it computes (all in float64; bf16 / fp32 inputs are widened exactly and are
never re-rounded), for each of the B sequences of a call:

  1. target logits  L[r, :] = (x_r . W) / T  for the M+1 embedding rows, and the
     target distributions p_{r+1} = softmax(L[r, :])          (Sec. 3.1, Eq. 2)
  2. draft distributions q_{j+1} from the draft model           (Sec. 3.1, Eq. 3)
  3. the standard accept test  eps < p[c] / q[c]                (Sec. 3.1, Eq. 4)
  4. the judge test  sigmoid(f_judge(e)) > delta  on the embedding of the judged
     token itself, f_judge linear                               (Sec. 4.1, "Model
     design" and "Inference"; App. B.1)
  5. z = z_stand OR z_judge                                     (Sec. 4.1, "Inference")
  6. accepted prefix = leading ones of z                        (Eq. 4; App. B.2, Fig. 8)
  7. one new token: from the residual norm(max(0, p - q)) at the first rejected
     position, or from p_{M+1} when everything was accepted     (Sec. 3.1, paragraph
     after Eq. 4; residual form after Chen et al. 2023, which the paper cites for
     the distribution-preservation guarantee)

Row convention (0-based): embedding row r of a sequence belongs to token
[s_L, c_1, ..., c_M][r] (Fig. 4, right).  Row r through the LM head gives the
paper's p_{r+1}.  Draft slot j holds c_{j+1}, q_{j+1}, eps_{j+1}: its standard
test reads LM-head row j, its judge test reads embedding row j+1.

Readings taken where the paper is silent (each is listed in the design notes):
  * the accept comparison is strict and evaluated without a division:
    accept iff eps * q[c] < p[c];
  * the judge comparison is done on the logit: g > log(delta / (1 - delta)),
    delta = 1 giving +inf (never accept), so that "delta = 1 reduces to SD";
  * uniforms[b, 0:M] are the accept draws, uniforms[b, M] is the one sampler draw;
  * inverse CDF in ascending token id on the unnormalised mass:
    next = min{ v : cumsum(res)[v] > u_s * sum(res) };
  * token ids outside [0, V) reject the slot and raise a status bit.

8-bit weights (the paper runs its targets with 8-bit weights: Table 1, App. B.3): ``W`` may hold FP8
E4M3 codes (uint8, the OCP "e4m3fn" format: 4 exponent bits with bias 7, 3 mantissa bits, no
infinities, 0x7f / 0xff = NaN) with one float32 scale per vocabulary entry; the effective weight is
scale[v] * decode(code), exactly, and everything downstream is unchanged.  ``W`` of dtype int8 is
8-bit integer weight-only quantisation with the same per-entry scales: decode(code) = the integer.

Variants of the rule that the paper itself uses (selected by ``rule`` / ``resample``):
  * top-K verification, the training-free baseline of Sec. 5: c is accepted iff it is among
    the K most probable tokens of p (K = V accepts every draft token, K = 1 is greedy
    matching as in Sec. 3.2); the target then decodes greedily, so the replacement or bonus
    token is argmax p.  Ties are ordered by token id (lower id ranks first).
  * ``resample = RESAMPLE_TARGET``: the literal "sample a correct token from p_i" of
    Sec. 3.1, i.e. the replacement is drawn from p_i itself instead of the residual.

Pre-norm wiring (Sec. 4.1, "Model design and training": the judge reads the last target embedding
*before* the final RMS normalisation, the LM head reads it after): ``rmsnorm_rows`` turns pre-norm
hidden states h into the LM-head input x = round_model_dtype(h * gamma / sqrt(mean(h^2) + eps)),
computed in float64 and rounded ONCE to the storage type of the embeddings (bf16 bit patterns, or
float32); ``verify(emb=rmsnorm_rows(h, ...), emb_judge=h)`` is then the paper's wiring.  The rounding
is part of the definition: the LM head multiplies bf16 operands, so the rounded tensor is what both
sides must use for the integer outputs to be comparable.

Parity pins for every function here live in tests/test_oracle_pins.py: the
paper's rule on hand cases, brute-force enumeration at V = 8 / M = 3, a
Monte-Carlo chi-square that standard-only verification emits the target
distribution, residual invariants, and textbook/library reductions.
"""

from __future__ import annotations

import math
from typing import Dict, Iterable, Optional, Sequence

import numpy as np

STATUS_BAD_TOKEN = 1      # a draft token id was outside [0, V)
STATUS_NAN = 2            # a NaN in target logits, draft row or judge logit, or a row that is no distribution
STATUS_ZERO_RESIDUAL = 4  # residual mass was exactly zero; fell back to sampling from p

MODE_JUDGE = 0     # z = z_stand OR z_judge
MODE_STANDARD = 1  # z = z_stand

RULE_SAMPLING = 0  # Eq. 4 with residual resampling
RULE_TOPK = 1      # accept iff c is among the K most probable target tokens; new token = argmax

RESAMPLE_RESIDUAL = 0  # replacement drawn from norm(max(0, p - q))
RESAMPLE_TARGET = 1    # replacement drawn from p itself

DRAFT_LOGITS = 0   # draft tensor holds fp32 logits (softmaxed here at temperature 1)
DRAFT_PROBS = 1    # draft tensor holds the probability vectors q_i themselves

_W_CHUNK_ROWS = 2048  # vocabulary rows widened to float64 at a time (memory bound only)


# --------------------------------------------------------------------------- helpers

def _e4m3fn_table() -> np.ndarray:
    """The 256 values of the FP8 E4M3 ("fn") format, written out from its definition."""
    t = np.empty(256, dtype=np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e, m = (code >> 3) & 0xF, code & 0x7
        if e == 0xF and m == 0x7:
            t[code] = np.nan
        elif e == 0:
            t[code] = sign * m * 2.0 ** -9            # subnormal: (m / 8) * 2^(1 - 7)
        else:
            t[code] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return t


E4M3FN = _e4m3fn_table()


def widen(x: np.ndarray) -> np.ndarray:
    """Exact float64 view of an input tensor: uint16 arrays are bf16 bit patterns, uint8 arrays
    are FP8 E4M3 codes, int8 arrays are 8-bit integer weights."""
    x = np.asarray(x)
    if x.dtype == np.uint8:
        return E4M3FN[x]
    if x.dtype == np.int8:
        return x.astype(np.float64)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if x.dtype in (np.float32, np.float64):
        return x.astype(np.float64)
    raise TypeError(f"unsupported input dtype {x.dtype}")


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float64 values to bfloat16 (8 significant bits, round-to-nearest-even, subnormals kept)
    and return the 16-bit patterns.  Written from the format: x = m * 2^e with 0.5 <= |m| < 1 is
    rounded to a multiple of 2^(e-8), or of 2^-133 (the smallest subnormal) below the normal range.
    Scaling by powers of two and rint are exact in float64, so there is no double rounding."""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)
    quantum_exp = np.maximum(e - 8, -133)                 # exponent of the spacing around x
    q = np.rint(np.ldexp(x, -quantum_exp))                # ties to even, exact
    y = np.ldexp(q, quantum_exp)
    y = np.where(np.abs(y) >= 2.0 ** 128, np.copysign(np.inf, x), y)   # beyond the largest finite bf16
    y = np.where(np.isnan(x), np.nan, y)
    f = y.astype(np.float32)                              # exact: every bf16 value is a float32
    bits = (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    return np.where(x == 0, (np.signbit(x).astype(np.uint16) << np.uint16(15)), bits).astype(np.uint16)


def rmsnorm_rows(hidden: np.ndarray, gamma: np.ndarray, eps: float):
    """Final RMS normalisation of pre-norm hidden states, row by row (Sec. 4.1, "Model design and
    training"): x[k] = h[k] * gamma[k] / sqrt(mean_k(h[k]^2) + eps) in float64, then rounded once to
    the storage type of ``hidden`` (uint16 = bf16 bit patterns -> bf16 bit patterns; float32 ->
    float32).  Returns (x in storage type, 1 / sqrt(mean + eps) per row as float64)."""
    h = widen(hidden)
    g = widen(gamma)
    inv = 1.0 / np.sqrt(np.mean(h * h, axis=-1) + float(eps))
    x = h * g * inv[..., None]
    hidden = np.asarray(hidden)
    if hidden.dtype == np.uint16:
        return round_to_bf16_bits(x), inv
    if hidden.dtype == np.float32:
        return x.astype(np.float32), inv
    raise TypeError(f"unsupported hidden-state dtype {hidden.dtype}")


def judge_threshold(delta: float) -> float:
    """logit(delta): sigmoid(g) > delta  <=>  g > log(delta / (1 - delta))  (Sec. 4.1)."""
    if not (0.5 <= delta <= 1.0):
        raise ValueError("delta must lie in [0.5, 1]")
    if delta == 1.0:
        return math.inf
    return math.log(delta / (1.0 - delta))


def softmax_rows(L: np.ndarray):
    """Row-wise softmax of float64 logits.  Returns (P, rowmax, rowsumexp)."""
    m = np.max(L, axis=-1, keepdims=True)
    e = np.exp(L - m)
    s = np.sum(e, axis=-1, keepdims=True)
    return e / s, m[..., 0], s[..., 0]


def target_logits(emb_rows: np.ndarray, W: np.ndarray, temperature: float = 1.0,
                  w_layout: str = "vd", w_scale: Optional[np.ndarray] = None) -> np.ndarray:
    """L[r, v] = sum_k x[r, k] * W[k, v] / T in float64 (W[k, v] scaled by w_scale[v] if given).

    ``W`` is stored [V, d] ("vd": row v is the vocabulary entry v) or [d, V] ("dv").
    The product is formed vocabulary-chunk by vocabulary-chunk only so that the
    float64 copy of W never has to exist at once; every L[r, v] is still one
    independent length-d dot product.
    """
    X = widen(emb_rows)
    if w_layout == "vd":
        V = W.shape[0]
    elif w_layout == "dv":
        V = W.shape[1]
    else:
        raise ValueError("w_layout must be 'vd' or 'dv'")
    L = np.empty((X.shape[0], V), dtype=np.float64)
    for v0 in range(0, V, _W_CHUNK_ROWS):
        v1 = min(V, v0 + _W_CHUNK_ROWS)
        Wc = widen(W[v0:v1]) if w_layout == "vd" else widen(W[:, v0:v1]).T
        L[:, v0:v1] = X @ Wc.T
    if w_scale is not None:
        L *= np.asarray(w_scale, dtype=np.float64)[None, :]
    if temperature != 1.0:
        L /= float(temperature)
    return L


def accept_standard(u: float, p_c: float, q_c: float) -> bool:
    """Eq. 4 for one slot: accept iff eps < p[c]/q[c], written as eps*q[c] < p[c]."""
    return bool(u * q_c < p_c)


def accepted_prefix(z: Sequence[int]) -> int:
    """Number of leading ones of the combined mask (Eq. 4; App. B.2, Fig. 8)."""
    m = 0
    for zj in z:
        if not zj:
            break
        m += 1
    return m


def residual(p_row: np.ndarray, q_row: np.ndarray) -> np.ndarray:
    """Unnormalised residual max(0, p - q) used after the first rejection."""
    return np.maximum(0.0, p_row - q_row)


def inverse_cdf(mass: np.ndarray, u: float):
    """Smallest token id v with cumsum(mass)[v] > u * sum(mass).

    Returns (token, margin) where margin is the distance from the threshold to the
    nearest edge of the chosen CDF interval, relative to the total mass.
    """
    S = float(np.sum(mass))
    cdf = np.cumsum(mass)
    thresh = float(u) * S
    hit = np.nonzero(cdf > thresh)[0]
    if hit.size:
        v = int(hit[0])
    else:  # rounding left the threshold at/above the last edge
        pos = np.nonzero(mass > 0)[0]
        v = int(pos[-1]) if pos.size else 0
    up = float(cdf[v]) - thresh
    lo = thresh - float(cdf[v - 1]) if v > 0 and cdf[v - 1] > 0 else math.inf
    margin = min(abs(up), abs(lo)) / S if S > 0 else 0.0
    return v, margin


def rank_of(logits_row: np.ndarray, c: int) -> int:
    """Number of tokens that rank before c: strictly larger logit, or equal logit and lower id."""
    lc = logits_row[c]
    return int(np.sum(logits_row > lc) + np.sum(logits_row[:c] == lc))


def topk_margin(logits_row: np.ndarray, c: int, k: int) -> float:
    """Distance (in logit units) of c from the top-K boundary: how far L[c] is from the logit
    that would have to overtake it (accepted) or that it would have to overtake (rejected)."""
    V = logits_row.shape[0]
    others = np.delete(logits_row, c)
    srt = np.sort(others)[::-1]                 # the other V-1 logits, descending
    if rank_of(logits_row, c) < k:              # accepted: the k-th largest of the others must pass it
        return float(logits_row[c] - srt[k - 1]) if k - 1 < V - 1 else math.inf
    return float(srt[k - 1] - logits_row[c])    # rejected: it must pass the k-th largest of the others


def argmax_lowest_id(logits_row: np.ndarray):
    """(argmax with lowest id among ties, runner-up id, gap between the two largest logits)."""
    v = int(np.argmax(logits_row))              # numpy returns the first maximum
    if logits_row.shape[0] == 1:
        return v, -1, math.inf
    rest = logits_row.copy(); rest[v] = -np.inf
    r = int(np.argmax(rest))
    return v, r, float(logits_row[v] - logits_row[r])


def mass_neighbours(mass: np.ndarray, v: int):
    """Nearest tokens below / above v that carry mass (-1 if none).  A sampler draw whose
    threshold sits within rounding of a CDF edge can only move to one of these."""
    below = np.nonzero(mass[:v] > 0)[0]
    above = np.nonzero(mass[v + 1:] > 0)[0]
    return (int(below[-1]) if below.size else -1), (int(above[0]) + v + 1 if above.size else -1)


def new_token(L: np.ndarray, P: np.ndarray, Q: np.ndarray, m: int, M: int, u_s: float, rule: int = RULE_SAMPLING,
              resample: int = RESAMPLE_RESIDUAL):
    """Step 7 for one sequence whose accepted prefix is m (Sec. 3.1, paragraph after Eq. 4): the
    replacement token from norm(max(0, p_{m+1} - q_{m+1})) if m < M, the bonus token from p_{M+1} if
    m == M; under RULE_TOPK the greedy token argmax p (lowest id on ties).  L, P are the M+1 target
    logit / probability rows, Q the M draft probability rows.
    Returns (token, margin, neighbour below, neighbour above, status bits)."""
    status = 0
    if rule == RULE_TOPK:                                      # greedy target: argmax of row m
        tok, runner_up, smargin = argmax_lowest_id(L[m])
        return tok, smargin, -1, runner_up, status
    if m < M and resample == RESAMPLE_RESIDUAL:
        mass = residual(P[m], Q[m])
        if np.sum(mass) == 0:
            status |= STATUS_ZERO_RESIDUAL
            mass = P[m]
    else:
        mass = P[m]                                            # bonus row, or "sample from p_i"
    tok, smargin = inverse_cdf(mass, u_s)
    below, above = mass_neighbours(mass, tok)
    return tok, smargin, below, above, status


def new_token_for_prefix(emb, W, draft, uniforms, b: int, m: int, *, draft_kind: int = DRAFT_LOGITS,
                         temperature: float = 1.0, w_layout: str = "vd", rule: int = RULE_SAMPLING,
                         resample: int = RESAMPLE_RESIDUAL, w_scale: Optional[np.ndarray] = None):
    """Step 7 alone, for sequence b with a GIVEN accepted prefix m (0 <= m <= M): what ``verify`` would
    emit as the new token had its masks produced that prefix.  The comparison uses it where a mask bit
    inside a near-tie band moved the library's prefix: the library's token must then still be the right
    one for its own prefix.  Returns (token, margin, neighbour below, neighbour above)."""
    emb = np.asarray(emb)
    M = emb.shape[1] - 1
    if not (0 <= m <= M):
        raise ValueError("prefix outside [0, M]")
    L = target_logits(emb[b, m:m + 1], W, temperature, w_layout, w_scale)       # only row m is needed
    P = softmax_rows(L)[0]
    Q = np.zeros((1, L.shape[1]))
    if m < M:
        Dm = np.asarray(draft[b, m:m + 1], dtype=np.float64)
        Q = softmax_rows(Dm)[0] if draft_kind == DRAFT_LOGITS else Dm
    # rows re-indexed so that row 0 is row m; M - m > 0 iff a draft row exists
    tok, margin, below, above, _ = new_token(L, P, Q, 0, 1 if m < M else 0, float(uniforms[b, M]), rule, resample)
    return tok, margin, below, above


# --------------------------------------------------------------------------- main entry

def verify(emb: np.ndarray, W: np.ndarray, w_judge: np.ndarray,
           draft_tokens: np.ndarray, draft: np.ndarray, uniforms: np.ndarray,
           *, emb_judge: Optional[np.ndarray] = None,
           mode: int = MODE_JUDGE, draft_kind: int = DRAFT_LOGITS,
           temperature: float = 1.0, delta: float = 0.5, judge_bias: float = 0.0,
           w_layout: str = "vd", seqs: Optional[Iterable[int]] = None,
           return_probs: bool = False, rule: int = RULE_SAMPLING, top_k: int = 1,
           resample: int = RESAMPLE_RESIDUAL, w_scale: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """Verify one batch of drafts.  See the module docstring for the steps.

    emb          [B, M+1, d]  LM-head input (bf16 bits as uint16, or float32)
    W            [V, d] / [d, V]  (float32, bf16 bits as uint16, FP8 E4M3 codes as uint8, or int8 weights)
    w_scale      [V] float32 per-vocabulary-entry scale of W (None = 1), meant for 8-bit weights
    w_judge      [d]
    draft_tokens [B, M] int
    draft        [B, rows >= M, V] float32 logits or probabilities (rows beyond M unused)
    uniforms     [B, M+1]
    seqs         optional subset of sequence indices to evaluate (sequences are
                 independent, so a subset is exact); outputs then have len(seqs) rows
    rule, top_k  RULE_SAMPLING (Eq. 4) or RULE_TOPK with 1 <= top_k <= V (Sec. 5 baseline)
    resample     RESAMPLE_RESIDUAL or RESAMPLE_TARGET (only read under RULE_SAMPLING)

    Under RULE_TOPK ``accept_margin`` holds the logit distance from the top-K boundary,
    ``sampler_margin`` the gap between the two largest logits of the decoded row and
    ``next_above`` the runner-up token.
    """
    emb = np.asarray(emb)
    B, Mp1, d = emb.shape
    M = Mp1 - 1
    seq_ids = list(range(B)) if seqs is None else [int(b) for b in seqs]
    nb = len(seq_ids)
    V = W.shape[0] if w_layout == "vd" else W.shape[1]
    thr = judge_threshold(delta)
    wj = widen(w_judge)
    ej_src = emb if emb_judge is None else np.asarray(emb_judge)
    if rule == RULE_TOPK and not (1 <= top_k <= V):
        raise ValueError("top_k must lie in [1, V]")

    out = {
        "accept_len": np.zeros(nb, np.int32), "next_token": np.zeros(nb, np.int32),
        "status": np.zeros(nb, np.uint32),
        "z_stand": np.zeros((nb, M), np.uint8), "z_judge": np.zeros((nb, M), np.uint8),
        "p_at_draft": np.zeros((nb, M)), "q_at_draft": np.zeros((nb, M)),
        "judge_logit": np.zeros((nb, M)),
        "row_max": np.zeros((nb, M + 1)), "row_sumexp": np.zeros((nb, M + 1)),
        "accept_margin": np.full((nb, M), np.inf), "judge_margin": np.full((nb, M), np.inf),
        "sampler_margin": np.zeros(nb),
        "next_below": np.full(nb, -1, np.int32), "next_above": np.full(nb, -1, np.int32),
    }
    if return_probs:
        out["probs"] = np.zeros((nb, M + 1, V))

    # step 1 for all selected rows at once (one float64 matmul per vocabulary chunk)
    L_all = target_logits(emb[seq_ids].reshape(nb * (M + 1), d), W, temperature, w_layout, w_scale)
    L_all = L_all.reshape(nb, M + 1, V)

    for i, b in enumerate(seq_ids):
        status = 0
        L = L_all[i]
        P, rmax, rsum = softmax_rows(L)                        # step 1: p_1 .. p_{M+1}
        if np.isnan(L).any():
            status |= STATUS_NAN
        Dm = np.asarray(draft[b, :M], dtype=np.float64)        # step 2: q_1 .. q_M
        if np.isnan(Dm).any():
            status |= STATUS_NAN
        Q = softmax_rows(Dm)[0] if draft_kind == DRAFT_LOGITS else Dm
        if np.isnan(Q).any() or np.isnan(P).any():             # e.g. a row without one finite logit: no distribution
            status |= STATUS_NAN
        E = widen(ej_src[b])                                   # judge input rows
        z = []
        for j in range(M):
            c = int(draft_tokens[b, j])
            g = float(np.dot(wj, E[j + 1])) + float(judge_bias)    # step 4: f_judge(e_{j+1})
            if math.isnan(g):
                status |= STATUS_NAN
            out["judge_logit"][i, j] = g
            if 0 <= c < V:
                p_c, q_c = float(P[j, c]), float(Q[j, c])
                u = float(uniforms[b, j])
                if rule == RULE_TOPK:                              # Sec. 5: among the K most probable
                    zs = rank_of(L[j], c) < top_k
                    out["accept_margin"][i, j] = topk_margin(L[j], c, top_k)
                else:
                    zs = accept_standard(u, p_c, q_c)              # step 3
                    out["accept_margin"][i, j] = abs(p_c / q_c - u) if q_c > 0 else math.inf
                zj = bool(g > thr)
                out["p_at_draft"][i, j], out["q_at_draft"][i, j] = p_c, q_c
                out["judge_margin"][i, j] = abs(g - thr)
            else:                                                  # invalid id: reject outright
                status |= STATUS_BAD_TOKEN
                zs, zj = False, False
            out["z_stand"][i, j], out["z_judge"][i, j] = zs, zj
            z.append(zs or (mode == MODE_JUDGE and zj))            # step 5
        m = accepted_prefix(z)                                     # step 6
        tok, smargin, below, above, st7 = new_token(L, P, Q, m, M, float(uniforms[b, M]), rule, resample)   # step 7
        status |= st7
        out["accept_len"][i], out["next_token"][i], out["status"][i] = m, tok, status
        out["row_max"][i], out["row_sumexp"][i] = rmax, rsum
        out["sampler_margin"][i] = smargin
        out["next_below"][i], out["next_above"][i] = below, above
        if return_probs:
            out["probs"][i] = P
    return out


# --------------------------------------------------------------------------- scalar tier

def append_tokens(token_buf: np.ndarray, lengths: np.ndarray, draft_tokens: np.ndarray, accept_len: np.ndarray,
                  next_token: np.ndarray) -> None:
    """The step after verification (Sec. 3.1, end of the paragraph after Eq. 4): the accepted draft
    tokens c_1..c_m* and the one new token are added to the sequence's context.  In place on
    token_buf [B, cap] / lengths [B]; tokens that do not fit into cap are dropped and the length
    saturates at cap."""
    B, cap = token_buf.shape
    for b in range(B):
        new = [int(t) for t in draft_tokens[b, :int(accept_len[b])]] + [int(next_token[b])]
        for t in new:
            if lengths[b] < cap:
                token_buf[b, lengths[b]] = t
                lengths[b] += 1


def verify_scalar(emb, W, w_judge, draft_tokens, draft, uniforms, *, mode=MODE_JUDGE,
                  draft_kind=DRAFT_LOGITS, temperature=1.0, delta=0.5, judge_bias=0.0):
    """The same definition written as plain Python loops over scalars.

    Only for tiny shapes (it is O(B * M * d * V) interpreted operations); used to
    check that the vectorised tier above did not mis-index anything.  W is [V, d].
    Returns (accept_len, next_token, z_stand, z_judge) as Python lists.
    """
    emb = widen(emb); W = widen(W); wj = widen(w_judge)
    B, Mp1, d = emb.shape
    M = Mp1 - 1
    V = W.shape[0]
    thr = judge_threshold(delta)

    def softmax_list(logits):
        mx = max(logits)
        ex = [math.exp(l - mx) for l in logits]
        s = 0.0
        for e in ex:
            s += e
        return [e / s for e in ex]

    acc, nxt, zs_all, zj_all = [], [], [], []
    for b in range(B):
        P = []
        for r in range(M + 1):
            logits = []
            for v in range(V):
                a = 0.0
                for k in range(d):
                    a += float(emb[b, r, k]) * float(W[v, k])
                logits.append(a / temperature)
            P.append(softmax_list(logits))
        Q = []
        for j in range(M):
            row = [float(x) for x in draft[b, j]]
            Q.append(softmax_list(row) if draft_kind == DRAFT_LOGITS else row)
        zs_row, zj_row, m, open_prefix = [], [], 0, True
        for j in range(M):
            c = int(draft_tokens[b, j])
            g = judge_bias
            for k in range(d):
                g += float(wj[k]) * float(emb[b, j + 1, k])
            zs = float(uniforms[b, j]) * Q[j][c] < P[j][c]
            zj = g > thr
            zs_row.append(int(zs)); zj_row.append(int(zj))
            if open_prefix and (zs or (mode == MODE_JUDGE and zj)):
                m += 1
            else:
                open_prefix = False
        if m < M:
            mass = [max(0.0, P[m][v] - Q[m][v]) for v in range(V)]
        else:
            mass = P[M]
        S = 0.0
        for x in mass:
            S += x
        thresh = float(uniforms[b, M]) * S
        run, tok = 0.0, None
        for v in range(V):
            run += mass[v]
            if run > thresh:
                tok = v
                break
        if tok is None:
            tok = max(v for v in range(V) if mass[v] > 0)
        acc.append(m); nxt.append(tok); zs_all.append(zs_row); zj_all.append(zj_row)
    return acc, nxt, zs_all, zj_all
