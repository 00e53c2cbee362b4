"""Element-by-element comparison of the HIP library's outputs with the oracle's.

TEST INFRASTRUCTURE ONLY (used by tests/, the smoke check and the benchmark's parity
line).  Takes two dicts of numpy arrays and applies the parity bar:

  * accept_len and next_token bit-exact, except
      - slots where |p/q - eps| < 1e-5 or the judge logit is within 1e-4 of its
        threshold (a flipped mask bit there is counted, not failed; the sequence's
        accept_len then follows from the library's own masks, and its next_token is held
        to what the oracle's step 7 gives for THAT prefix when the caller supplies
        ``replay``, and left unchecked otherwise),
      - sampler draws whose threshold lies within SAMPLER_BAND of a CDF edge, and only
        if the other side returned the neighbouring token that carries mass;
  * p and q at the drafted tokens, row sum-exp and (if present) the full softmax within
    2e-3 relative; row max within 1e-3 absolute.  The library's probabilities are float32: below
    float32's smallest normal number (2^-126) that type carries no relative precision, so there the
    check is that the library's value is below that bound as well;
  * judge logits within 1e-3 absolute;
  * status words equal.
"""

from __future__ import annotations

from typing import Callable, Dict, Optional, Tuple

import numpy as np

ACCEPT_BAND = 1e-5
TOPK_BAND = 1e-4      # logit distance from the top-K boundary / between the two largest logits
JUDGE_BAND = 1e-4
SAMPLER_BAND = 1e-5
REL_TOL = 2e-3
F32_MIN_NORMAL = 2.0 ** -126   # smallest normal float32: relative precision ends here
JUDGE_ABS_TOL = 1e-3


def compare(gpu: Dict[str, np.ndarray], ref: Dict[str, np.ndarray], mode_judge: bool = True,
            rule_topk: bool = False,
            replay: Optional[Callable[[int, int], Tuple[int, float, int, int]]] = None) -> Dict[str, int]:
    """Raise AssertionError on any violation; return counts of excused near-ties.

    ``replay(b, m)`` (optional) returns the oracle's (token, margin, neighbour below, neighbour above)
    for row b of these dicts under a forced accepted prefix m (verify_oracle.new_token_for_prefix); with
    it, a sequence whose masks differ inside a band still has its next_token checked.

    With ``rule_topk`` the oracle's accept_margin / sampler_margin are logit distances (top-K
    boundary, gap between the two largest logits) and the band is TOPK_BAND for both."""
    accept_band = TOPK_BAND if rule_topk else ACCEPT_BAND
    sampler_band = TOPK_BAND if rule_topk else SAMPLER_BAND
    B, M = ref["z_stand"].shape
    rep = {"slots": B * M, "sequences": B, "near_tie_stand": 0, "near_tie_judge": 0, "near_tie_sampler": 0,
           "excluded_sequences": 0, "mismatch": 0}
    status_gpu = gpu["status"].astype(np.int64) & 0xFFFFFFFF
    assert np.array_equal(status_gpu, ref["status"].astype(np.int64)), (status_gpu, ref["status"])
    clean = ref["status"] == 0

    zs_diff = gpu["z_stand"].astype(bool) != ref["z_stand"].astype(bool)
    zj_diff = gpu["z_judge"].astype(bool) != ref["z_judge"].astype(bool)
    bad_s = zs_diff & ~(ref["accept_margin"] < accept_band)
    bad_j = zj_diff & ~(ref["judge_margin"] < JUDGE_BAND)
    assert not bad_s.any(), f"z_stand differs outside the band at {np.argwhere(bad_s).tolist()}"
    assert not bad_j.any(), f"z_judge differs outside the band at {np.argwhere(bad_j).tolist()}"
    rep["near_tie_stand"] = int(zs_diff.sum())
    rep["near_tie_judge"] = int(zj_diff.sum())

    z_gpu = gpu["z_stand"].astype(bool) | (gpu["z_judge"].astype(bool) if mode_judge else False)
    z_ref = ref["z_stand"].astype(bool) | (ref["z_judge"].astype(bool) if mode_judge else False)
    for b in range(B):
        # the library's own prefix must be the leading ones of its own masks, always
        lead = int(np.argmin(np.append(z_gpu[b], False)))
        assert int(gpu["accept_len"][b]) == lead, (b, gpu["accept_len"][b], z_gpu[b])
        r, margin = int(ref["next_token"][b]), float(ref["sampler_margin"][b])
        nbrs = (int(ref["next_below"][b]), int(ref["next_above"][b]))
        if (z_gpu[b] != z_ref[b]).any():
            # a mask bit inside a band went the other way (checked above): the library's prefix is the one of its
            # own masks (checked above); its token must be right for that prefix
            rep["excluded_sequences"] += 1
            if replay is None or not clean[b]:
                continue
            r, margin, lo, hi = replay(b, lead)
            nbrs = (int(lo), int(hi))
            rep["replayed_sequences"] = rep.get("replayed_sequences", 0) + 1
        else:
            assert int(gpu["accept_len"][b]) == int(ref["accept_len"][b]), (b, gpu["accept_len"][b], ref["accept_len"][b])
        g = int(gpu["next_token"][b])
        if g != r:
            near = margin < sampler_band and g >= 0 and g in nbrs
            assert near, f"next_token differs at b={b}: {g} vs {r}, margin {margin:.3e}"
            rep["near_tie_sampler"] += 1

    def rel_close(name, a, r, mask=None):
        a = np.asarray(a, dtype=np.float64); r = np.asarray(r, dtype=np.float64)
        if mask is not None:
            a, r = a[mask], r[mask]
        tiny = np.abs(r) < F32_MIN_NORMAL
        assert (np.abs(a[tiny]) <= F32_MIN_NORMAL * (1 + REL_TOL)).all(), f"{name}: not tiny where the oracle's value is"
        a, r = a[~tiny], r[~tiny]
        err = np.abs(a - r) / np.abs(r)
        assert (err <= REL_TOL).all(), f"{name}: max rel err {err.max():.3e}"
        return float(err.max()) if err.size else 0.0

    ok_rows = np.repeat(clean[:, None], M, axis=1)
    valid = ok_rows & (ref["p_at_draft"] > 0)
    rep["max_rel_p"] = rel_close("p_at_draft", gpu["p_at_draft"], ref["p_at_draft"], valid)
    rep["max_rel_q"] = rel_close("q_at_draft", gpu["q_at_draft"], ref["q_at_draft"], valid)
    jerr = np.abs(gpu["judge_logit"].astype(np.float64) - ref["judge_logit"])[ok_rows]
    assert (jerr <= JUDGE_ABS_TOL).all(), f"judge_logit: max abs err {jerr.max():.3e}"
    rep["max_abs_judge"] = float(jerr.max()) if jerr.size else 0.0
    if "row_sumexp" in gpu:
        ok1 = np.repeat(clean[:, None], M + 1, axis=1)
        # (max, sumexp) pairs are only defined up to the max; compare log-sum-exp
        lse_g = gpu["row_max"].astype(np.float64) + np.log(gpu["row_sumexp"].astype(np.float64))
        lse_r = ref["row_max"] + np.log(ref["row_sumexp"])
        assert (np.abs(lse_g - lse_r)[ok1] <= REL_TOL).all(), "row log-sum-exp differs"
        assert (np.abs(gpu["row_max"] - ref["row_max"])[ok1] <= 1e-3).all(), "row_max differs"
    if "probs" in gpu and "probs" in ref:
        rep["max_rel_probs"] = rel_close("probs", gpu["probs"], ref["probs"], np.broadcast_to(clean[:, None, None], ref["probs"].shape))
    return rep
