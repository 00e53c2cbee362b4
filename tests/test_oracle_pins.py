"""Pins for the float64 oracle: things the paper and the mathematics fix, none of
which is computed by the oracle itself.

  * Eq. 4 on hand cases, the OR rule and the prefix cut (text fixtures)
  * exact integer arithmetic for the LM-head contraction (catches a transposed
    operand or a wrong index)
  * scipy / closed forms for softmax and the inverse CDF
  * brute-force enumeration at V = 8, M = 3 with every interval edge probed
  * Monte-Carlo chi-square: standard-only verification emits the target distribution
    (and the plausible wrong reading "resample from p" is shown to fail it)
  * residual invariants, special cases, judge row offset
  * acceptance statistics of the synthetic workloads against the closed form
    1 - TV(p, q) -> 2 Phi(-sigma / 2)
"""

import itertools
import math
import os

import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import verify_oracle as vo
from synth import VerifyShape, make_inputs, bf16_bits_from_f32, f32_from_bf16_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- builders

def direct_case(P_rows, Q_rows, judge_bits, tokens, uniforms, **kw):
    """Build oracle inputs whose target distributions are exactly softmax(log P_rows).

    d = V, W = identity, embeddings = float32(log P).  The judge reads a separate
    tensor whose row j+1 is (+1 | -1, 0, ...) with w_judge = e_0, so judge logits
    are +-1.  Draft is handed over as probabilities.
    """
    P_rows = np.asarray(P_rows, dtype=np.float64)
    Mp1, V = P_rows.shape
    M = Mp1 - 1
    tokens = np.asarray(tokens, dtype=np.int32).reshape(-1, M)
    B = tokens.shape[0]
    emb = np.broadcast_to(np.log(P_rows).astype(np.float32), (B, Mp1, V)).copy()
    W = np.eye(V, dtype=np.float32)
    ej = np.zeros((B, Mp1, V), dtype=np.float32)
    jb = np.asarray(judge_bits).reshape(-1, M)
    ej[:, 1:, 0] = np.where(np.broadcast_to(jb, (B, M)) > 0, 1.0, -1.0)
    ej[:, 0, 0] = 77.0  # row 0 must never be read by the judge
    wj = np.zeros(V, dtype=np.float32); wj[0] = 1.0
    Q = np.broadcast_to(np.asarray(Q_rows, dtype=np.float32), (B, M, V)).copy()
    u = np.asarray(uniforms, dtype=np.float32).reshape(B, Mp1)
    return vo.verify(emb, W, wj, tokens, Q, u, emb_judge=ej, draft_kind=vo.DRAFT_PROBS, **kw)


def py_softmax(logits):
    mx = max(logits)
    ex = [math.exp(x - mx) for x in logits]
    s = math.fsum(ex)
    return [e / s for e in ex]


def random_dist(rng, V, conc=1.0):
    x = rng.gamma(conc, size=V) + 1e-3
    return x / x.sum()


# ----------------------------------------------------------------------------- Eq. 4, OR, prefix

def test_eq4_hand_cases():
    # p >= q: accepted for every eps in [0, 1)
    for u in (0.0, 0.3, 0.999999, float(np.float32(1) - np.float32(2 ** -24))):
        assert vo.accept_standard(u, 0.6, 0.5)
        assert vo.accept_standard(u, 0.5, 0.5) == (u < 1.0)
    # p = q / 2: accepted iff eps < 1/2 (strict)
    assert vo.accept_standard(0.49999, 0.2, 0.4)
    assert not vo.accept_standard(0.5, 0.2, 0.4)
    assert not vo.accept_standard(0.50001, 0.2, 0.4)
    # q[c] = 0 corner: accept iff p[c] > 0, no NaN
    assert vo.accept_standard(0.9, 0.1, 0.0)
    assert not vo.accept_standard(0.0, 0.0, 0.0)


def _golden_cases():
    with open(os.path.join(GOLDEN, "mask_prefix_cases.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            lhs, rhs = line.split("->")
            zs, zj = lhs.split()
            z, m = rhs.split()
            yield [int(c) for c in zs], [int(c) for c in zj], [int(c) for c in z], int(m)


def test_prefix_and_or_fixture():
    rng = np.random.default_rng(5)
    n = 0
    for zs, zj, z, m in _golden_cases():
        n += 1
        M, V = len(zs), 8
        assert vo.accepted_prefix(z) == m
        # realise the masks through the full oracle: z_stand via p/q and eps
        P = np.stack([random_dist(rng, V) for _ in range(M + 1)])
        Q = np.stack([random_dist(rng, V) for _ in range(M)])
        toks, us = [], []
        for j in range(M):
            ratio = P[j] / Q[j].astype(np.float32).astype(np.float64)
            if zs[j]:
                c = int(np.argmax(ratio)); u = min(0.99, 0.5 * ratio[c])
            else:
                c = int(np.argmin(ratio)); assert ratio[c] < 0.9; u = 0.5 * (ratio[c] + 1.0)
            toks.append(c); us.append(u)
        out = direct_case(P, Q, zj, toks, us + [0.37])
        assert out["z_stand"][0].tolist() == zs
        assert out["z_judge"][0].tolist() == zj
        assert int(out["accept_len"][0]) == m
        # standard-only mode ignores the judge; OR can only add accepts
        std = direct_case(P, Q, zj, toks, us + [0.37], mode=vo.MODE_STANDARD)
        assert int(std["accept_len"][0]) == vo.accepted_prefix(zs) <= m
        # delta = 1 reduces to standard SD (Sec. 4.1)
        d1 = direct_case(P, Q, zj, toks, us + [0.37], delta=1.0)
        assert int(d1["accept_len"][0]) == int(std["accept_len"][0])
        assert int(d1["next_token"][0]) == int(std["next_token"][0])
        assert not d1["z_judge"].any()
    assert n >= 10


def test_judge_threshold_and_logit_form():
    assert vo.judge_threshold(0.5) == 0.0
    assert vo.judge_threshold(1.0) == math.inf
    for delta in (0.6, 0.9, 0.999):
        t = vo.judge_threshold(delta)
        # sigmoid(t) == delta and the comparison is monotone around it
        assert abs(scipy.special.expit(t) - delta) < 1e-15
        assert scipy.special.expit(t + 1e-9) > delta > scipy.special.expit(t - 1e-9)
    with pytest.raises(ValueError):
        vo.judge_threshold(0.4)


def test_judge_reads_row_of_the_judged_token():
    # Sec. 4.1: c_i is judged on its own embedding e_i; with rows [s_L, c_1..c_M]
    # that is row j+1 for slot j.  Only row j+1 carries a positive judge logit.
    V, M = 8, 4
    rng = np.random.default_rng(0)
    P = np.stack([random_dist(rng, V) for _ in range(M + 1)])
    Q = P[:M].copy()
    for target in range(M):
        bits = [1 if j == target else 0 for j in range(M)]
        out = direct_case(P, Q, bits, [0] * M, [0.5] * (M + 1))
        assert out["z_judge"][0].tolist() == bits
        assert np.allclose(out["judge_logit"][0], np.where(np.array(bits) > 0, 1.0, -1.0))
    # bias shifts the logit; threshold moves with delta
    out = direct_case(P, Q, [0] * M, [0] * M, [0.5] * (M + 1), judge_bias=1.5)
    assert out["z_judge"].all() and np.allclose(out["judge_logit"], 0.5)
    out = direct_case(P, Q, [1] * M, [0] * M, [0.5] * (M + 1), delta=0.75)  # logit(0.75)=1.0986 > 1
    assert not out["z_judge"].any()
    assert np.allclose(out["judge_margin"], math.log(3.0) - 1.0)


# ----------------------------------------------------------------------------- textbook reductions

def test_logits_exact_integer_arithmetic():
    # integer-valued operands: the contraction is exact, compare with Python ints
    rng = np.random.default_rng(1)
    R, d, V = 3, 7, 11
    X = rng.integers(-8, 9, size=(R, d)); W = rng.integers(-8, 9, size=(V, d))
    want = [[sum(int(X[r, k]) * int(W[v, k]) for k in range(d)) for v in range(V)] for r in range(R)]
    got = vo.target_logits(X.astype(np.float32), W.astype(np.float32))
    assert got.shape == (R, V) and np.array_equal(got, np.array(want, dtype=np.float64))
    got_dv = vo.target_logits(X.astype(np.float32), np.ascontiguousarray(W.T).astype(np.float32), w_layout="dv")
    assert np.array_equal(got_dv, got)
    got_T = vo.target_logits(X.astype(np.float32), W.astype(np.float32), temperature=2.0)
    assert np.array_equal(got_T, got / 2.0)


def test_bf16_widening_is_exact():
    bits = np.array([0x3F80, 0xBF80, 0x4049, 0x0000, 0x8000, 0x3DCD, 0x7F7F], dtype=np.uint16)
    want = [1.0, -1.0, 3.140625, 0.0, -0.0, 0.10009765625, 3.3895313892515355e38]
    assert vo.widen(bits).tolist() == want
    # chunked path must see every vocabulary row once (chunk edge at 2048)
    rng = np.random.default_rng(2)
    V, d = 2048 + 37, 16
    Wb = rng.integers(0x3C00, 0x4100, size=(V, d)).astype(np.uint16)
    x = np.zeros((1, d), dtype=np.float32); x[0, 3] = 1.0
    assert np.array_equal(vo.target_logits(x, Wb)[0], vo.widen(Wb)[:, 3])


def test_softmax_against_scipy():
    rng = np.random.default_rng(3)
    L = rng.normal(size=(5, 1000)) * 4.0
    L[2] += 700.0  # would overflow a naive exp
    P, m, s = vo.softmax_rows(L)
    assert np.allclose(P, scipy.special.softmax(L, axis=1), rtol=1e-12, atol=0)
    assert np.allclose(np.log(P), scipy.special.log_softmax(L, axis=1), rtol=0, atol=1e-12)
    assert np.allclose(P.sum(1), 1.0, atol=1e-12)
    assert np.array_equal(m, L.max(1))
    assert np.allclose(np.log(s) + m, scipy.special.logsumexp(L, axis=1), atol=1e-12)


def test_inverse_cdf_closed_forms():
    # uniform mass over V tokens: token = floor(u * V)
    V = 10
    for u in (0.0, 0.05, 0.1, 0.15, 0.95, 0.999999):
        tok, _ = vo.inverse_cdf(np.ones(V), u)
        # u*V exactly on an edge belongs to the upper token (cdf > thresh is strict)
        assert tok == int(math.floor(u * V + 1e-12))
    # zero-mass tokens are never returned, including at u = 0 and u -> 1
    mass = np.array([0.0, 0.0, 2.0, 0.0, 1.0, 0.0])
    assert vo.inverse_cdf(mass, 0.0)[0] == 2
    assert vo.inverse_cdf(mass, 0.66)[0] == 2
    assert vo.inverse_cdf(mass, 0.67)[0] == 4
    assert vo.inverse_cdf(mass, 1.0 - 2 ** -24)[0] == 4
    # searchsorted form on random mass; margin is the distance to the nearest edge
    rng = np.random.default_rng(4)
    mass = rng.random(257) * (rng.random(257) > 0.3)
    cdf = np.cumsum(mass); S = mass.sum()
    for u in rng.random(200):
        tok, margin = vo.inverse_cdf(mass, u)
        assert tok == int(np.searchsorted(cdf, u * S, side="right"))
        assert mass[tok] > 0 and 0 <= margin <= mass[tok] / S


# ----------------------------------------------------------------------------- residual

def test_residual_invariants():
    rng = np.random.default_rng(6)
    for _ in range(50):
        V = int(rng.integers(2, 200))
        p, q = random_dist(rng, V, 0.3), random_dist(rng, V, 0.3)
        r = vo.residual(p, q)
        assert (r >= 0).all()
        S = r.sum()
        assert abs(S - (1.0 - np.minimum(p, q).sum())) < 1e-12
        assert abs(S - np.maximum(0.0, q - p).sum()) < 1e-12
        assert abs((r / S).sum() - 1.0) < 1e-12
        # a token the standard test can reject has p < q, hence zero residual mass
        assert (r[p < q] == 0).all()


def test_rejected_token_is_never_reemitted():
    shape = VerifyShape("t", 32, 4, 32, 96, "f32", 1.5)
    for seed in range(3):
        x = make_inputs(shape, seed)
        out = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"],
                        x["uniforms"], mode=vo.MODE_STANDARD)
        rej = out["accept_len"] < shape.M
        assert rej.any()
        b = np.nonzero(rej)[0]
        assert (out["next_token"][b] != x["draft_tokens"][b, out["accept_len"][b]]).all()
        assert (out["status"] == 0).all()


# ----------------------------------------------------------------------------- brute force V=8, M=3

def _brute_setup():
    rng = np.random.default_rng(11)
    V, M = 8, 3
    P = np.stack([random_dist(rng, V, 0.7) for _ in range(M + 1)])
    Q = np.stack([random_dist(rng, V, 0.7) for _ in range(M)]).astype(np.float32)
    judge_bits = [0, 1, 0]
    # independent evaluation of what the oracle should see: p from float32 logits
    Pt = [py_softmax([float(x) for x in np.log(P[r]).astype(np.float32)]) for r in range(M + 1)]
    Qt = [[float(x) for x in Q[j]] for j in range(M)]
    return V, M, P, Q, judge_bits, Pt, Qt


def _mass_after(m, M, Pt, Qt, V):
    if m < M:
        return [max(0.0, Pt[m][v] - Qt[m][v]) for v in range(V)]
    return list(Pt[M])


def test_bruteforce_every_interval_edge():
    V, M, P, Q, jb, Pt, Qt = _brute_setup()
    eps = 1e-6  # probes sit this far inside each interval (float32 uniforms resolve 6e-8)
    toks, us, want_m, want_tok = [], [], [], []
    for c in itertools.product(range(V), repeat=M):
        a = [min(1.0, Pt[j][c[j]] / Qt[j][c[j]]) for j in range(M)]  # Pr[z_stand_j = 1]
        for m in range(M + 1):
            # force prefix length m: slots < m accepted (judge bit, or eps just inside),
            # slot m rejected (needs judge bit 0 and a < 1, eps just outside)
            if m < M and (jb[m] or a[m] >= 1.0 - 2 * eps):
                continue
            u = []
            for j in range(M):
                if j < m:
                    u.append(0.999 if jb[j] else max(0.0, a[j] - eps))
                    if not jb[j] and a[j] - eps <= 0.0:
                        break
                elif j == m:
                    u.append(a[j] + eps)
                else:
                    u.append(0.123)  # irrelevant after the cut
            if len(u) < M:
                continue
            mass = _mass_after(m, M, Pt, Qt, V)
            S = math.fsum(mass)
            edge = 0.0
            for v in range(V):
                lo, hi = edge / S, (edge + mass[v]) / S
                edge += mass[v]
                if hi - lo < 4 * eps:
                    continue
                for us_ in (lo + eps, hi - eps):
                    toks.append(c); us.append(u + [us_]); want_m.append(m); want_tok.append(v)
    assert len(toks) > 10000
    out = direct_case(P, Q, jb, toks, us)
    assert np.array_equal(out["accept_len"], np.array(want_m))
    assert np.array_equal(out["next_token"], np.array(want_tok))
    assert (out["status"] == 0).all()


def test_bruteforce_law_on_a_grid():
    # Law of (m*, next) for fixed drafts: Pr[z_j = 1] = 1 if judge bit else min(1, p/q);
    # Pr[next = v | m* = m] = mass_m[v] / S_m.  A midpoint grid over the four uniforms
    # must reproduce it to grid resolution.
    V, M, P, Q, jb, Pt, Qt = _brute_setup()
    G, GS = 8, 64
    mids = (np.arange(G) + 0.5) / G
    smid = (np.arange(GS) + 0.5) / GS
    grid = np.array([(a, b, c, s) for a in mids for b in mids for c in mids for s in smid])
    for c in [(0, 1, 2), (7, 7, 7), (3, 0, 5)]:
        out = direct_case(P, Q, jb, [c] * len(grid), grid)
        acc = [1.0 if jb[j] else min(1.0, Pt[j][c[j]] / Qt[j][c[j]]) for j in range(M)]
        for m in range(M + 1):
            pm = np.prod(acc[:m]) * ((1.0 - acc[m]) if m < M else 1.0)
            sel = out["accept_len"] == m
            assert abs(sel.mean() - pm) <= 1.5 / G
            if pm < 0.05:
                continue
            mass = _mass_after(m, M, Pt, Qt, V)
            S = math.fsum(mass)
            for v in range(V):
                emp = (out["next_token"][sel] == v).mean()
                assert abs(emp - mass[v] / S) <= 2.0 / GS


def test_vectorised_tier_matches_scalar_tier():
    for seed, kind in [(0, "f32"), (1, "bf16"), (2, "f32")]:
        shape = VerifyShape("t", 2, 3, 8, 32, kind, 1.0)
        x = make_inputs(shape, seed)
        for mode in (vo.MODE_JUDGE, vo.MODE_STANDARD):
            out = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"],
                            x["uniforms"], mode=mode)
            acc, nxt, zs, zj = vo.verify_scalar(x["emb"], x["W"], x["w_judge"], x["draft_tokens"],
                                                x["draft_logits"], x["uniforms"], mode=mode)
            assert out["accept_len"].tolist() == acc
            assert out["next_token"].tolist() == nxt
            assert out["z_stand"].tolist() == zs and out["z_judge"].tolist() == zj


# ----------------------------------------------------------------------------- Monte-Carlo

def _first_emitted(out, tokens):
    first = np.where(out["accept_len"] > 0, tokens[:, 0], out["next_token"])
    return first


def test_standard_verification_preserves_target_distribution():
    # Sec. 1 / Sec. 3.1: standard SD emits tokens distributed exactly as the target.
    # Draw c ~ q, eps, u_s many times; the first emitted token must follow p_1.
    rng = np.random.default_rng(2025)
    V, M, N = 8, 2, 120_000
    P = np.stack([random_dist(rng, V, 0.8) for _ in range(M + 1)])
    Q = np.stack([random_dist(rng, V, 0.8) for _ in range(M)]).astype(np.float32)
    q0 = Q[0].astype(np.float64); q0 /= q0.sum()
    Qn = Q.astype(np.float64) / Q.astype(np.float64).sum(1, keepdims=True)
    tokens = np.stack([rng.choice(V, size=N, p=Qn[j]) for j in range(M)], 1)
    u = rng.random((N, M + 1)).astype(np.float32)
    out = direct_case(P, Q, [0] * M, tokens, u, mode=vo.MODE_STANDARD)
    p1 = np.array(py_softmax([float(x) for x in np.log(P[0]).astype(np.float32)]))
    first = _first_emitted(out, tokens)
    counts = np.bincount(first, minlength=V)
    chi = scipy.stats.chisquare(counts, p1 * N)
    assert chi.pvalue > 0.01, chi
    # second emitted token given the first was accepted follows p_2
    sel = out["accept_len"] >= 1
    second = np.where(out["accept_len"][sel] > 1, tokens[sel, 1], out["next_token"][sel])
    p2 = np.array(py_softmax([float(x) for x in np.log(P[1]).astype(np.float32)]))
    chi2 = scipy.stats.chisquare(np.bincount(second, minlength=V), p2 * sel.sum())
    assert chi2.pvalue > 0.01, chi2
    # all accepted: the bonus token follows p_{M+1}
    full = out["accept_len"] == M
    p3 = np.array(py_softmax([float(x) for x in np.log(P[2]).astype(np.float32)]))
    chi3 = scipy.stats.chisquare(np.bincount(out["next_token"][full], minlength=V), p3 * full.sum())
    assert chi3.pvalue > 0.01, chi3

    # power of the test: resampling from plain p after a rejection (the wrong reading
    # of "sample a correct token from p_i") is rejected by the same statistic
    cdf = np.cumsum(p1)
    wrong = np.where(out["accept_len"] > 0, tokens[:, 0],
                     np.minimum(np.searchsorted(cdf, u[:, M].astype(np.float64) * cdf[-1], side="right"), V - 1))
    assert scipy.stats.chisquare(np.bincount(wrong, minlength=V), p1 * N).pvalue < 1e-6
    # and so is a rule with the ratio upside down (eps < q/p)
    flipped = u[:, 0] * p1[tokens[:, 0]] < q0[tokens[:, 0]]
    wrong2 = np.where(flipped, tokens[:, 0], out["next_token"])
    assert scipy.stats.chisquare(np.bincount(wrong2, minlength=V), p1 * N).pvalue < 1e-6


# ----------------------------------------------------------------------------- special cases

def _exact_logit_inputs(seed, B=3, M=4, d=16, V=40):
    """Embeddings / weights on a coarse dyadic grid so that logits are exact in float32."""
    rng = np.random.default_rng(seed)
    emb = (rng.integers(-8, 9, size=(B, M + 1, d)) / 8.0).astype(np.float32)
    W = (rng.integers(-8, 9, size=(V, d)) / 8.0).astype(np.float32)
    wj = (rng.integers(-8, 9, size=d) / 8.0).astype(np.float32)
    L = np.einsum("brk,vk->brv", emb.astype(np.float64), W.astype(np.float64))
    assert np.array_equal(L, L.astype(np.float32).astype(np.float64))
    tokens = rng.integers(0, V, size=(B, M)).astype(np.int32)
    return emb, W, wj, L.astype(np.float32), tokens


def test_identical_draft_accepts_everything():
    emb, W, wj, L32, tokens = _exact_logit_inputs(0)
    B, Mp1, _ = emb.shape
    for u_val in (0.0, 0.5, float(np.float32(1) - np.float32(2 ** -24))):
        u = np.full((B, Mp1), u_val, dtype=np.float32)
        out = vo.verify(emb, W, wj, tokens, L32, u, mode=vo.MODE_STANDARD)
        assert (out["accept_len"] == Mp1 - 1).all()
        assert out["z_stand"].all()
        assert np.array_equal(out["p_at_draft"], out["q_at_draft"])


def test_huge_judge_bias_gives_bonus_token_from_last_row():
    emb, W, wj, L32, tokens = _exact_logit_inputs(1)
    B, Mp1, _ = emb.shape
    rng = np.random.default_rng(9)
    D = (L32 + rng.normal(size=L32.shape) * 3).astype(np.float32)
    u = rng.random((B, Mp1)).astype(np.float32)
    out = vo.verify(emb, W, wj, tokens, D, u, judge_bias=1e6)
    assert (out["accept_len"] == Mp1 - 1).all() and out["z_judge"].all()
    for b in range(B):
        pM = scipy.special.softmax(L32[b, -1].astype(np.float64))
        want = int(np.searchsorted(np.cumsum(pM), float(u[b, -1]) * pM.sum(), side="right"))
        assert int(out["next_token"][b]) == want


def test_all_rejecting_case_gives_zero_prefix():
    emb, W, wj, L32, tokens = _exact_logit_inputs(2)
    B, Mp1, V = L32.shape
    D = L32.copy()
    for b in range(B):
        for j in range(Mp1 - 1):
            D[b, j, tokens[b, j]] += 5.0  # q[c] > p[c] at every drafted token
    u = np.full((B, Mp1), np.float32(1) - np.float32(2 ** -24), dtype=np.float32)
    out = vo.verify(emb, W, wj, tokens, D, u, judge_bias=-1e6)
    assert (out["accept_len"] == 0).all() and not out["z_stand"].any() and not out["z_judge"].any()
    assert (out["next_token"] != tokens[:, 0]).all()


def test_bad_token_and_nan_status():
    emb, W, wj, L32, tokens = _exact_logit_inputs(3)
    B, Mp1, V = L32.shape
    u = np.full((B, Mp1), 0.25, dtype=np.float32)
    tokens = tokens.copy(); tokens[1, 2] = V; tokens[2, 0] = -1
    Dn = (L32 + np.random.default_rng(0).normal(size=L32.shape)).astype(np.float32)
    out = vo.verify(emb, W, wj, tokens, Dn, u, judge_bias=1e6)
    assert out["status"].tolist() == [0, vo.STATUS_BAD_TOKEN, vo.STATUS_BAD_TOKEN]
    assert out["accept_len"].tolist() == [Mp1 - 1, 2, 0]
    # q == p at the cut leaves no residual mass: flagged, and the token comes from p
    out = vo.verify(emb, W, wj, tokens, L32, u, judge_bias=1e6)
    assert out["status"].tolist() == [0, vo.STATUS_BAD_TOKEN | vo.STATUS_ZERO_RESIDUAL] * 1 + \
        [vo.STATUS_BAD_TOKEN | vo.STATUS_ZERO_RESIDUAL]
    pm = scipy.special.softmax(L32[1, 2].astype(np.float64))
    assert int(out["next_token"][1]) == int(np.searchsorted(np.cumsum(pm), 0.25 * pm.sum(), side="right"))
    D = L32.copy(); D[0, 1, 5] = np.nan
    out = vo.verify(emb, W, wj, np.clip(tokens, 0, V - 1), D, u)
    assert out["status"][0] & vo.STATUS_NAN and not (out["status"][1:] & vo.STATUS_NAN).any()


def test_subset_of_sequences_is_exact():
    shape = VerifyShape("t", 6, 3, 16, 64, "bf16", 1.0)
    x = make_inputs(shape, 4)
    args = (x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"])
    full = vo.verify(*args, return_probs=True)
    part = vo.verify(*args, seqs=[4, 1], return_probs=True)
    for k in full:
        assert np.array_equal(part[k], full[k][[4, 1]]), k


# ----------------------------------------------------------------------------- workload statistics

@pytest.mark.parametrize("sigma,want", [(1.0, 0.617), (2.0, 0.326)])
def test_synthetic_acceptance_rate_matches_closed_form(sigma, want):
    # draft logits = target logits + sigma * N(0,1) iid over a large vocabulary gives a
    # per-slot standard acceptance probability 1 - TV(p, q) -> 2 Phi(-sigma/2)
    # (0.617 at sigma = 1; at V = 1024 the finite-vocabulary value for sigma = 2 is 0.326).
    shape = VerifyShape("t", 64, 5, 64, 1024, "f32", sigma)
    acc, n, jacc = 0, 0, 0
    for seed in range(4):
        x = make_inputs(shape, seed)
        out = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"])
        acc += int(out["z_stand"].sum()); jacc += int(out["z_judge"].sum()); n += out["z_stand"].size
        assert (out["status"] == 0).all()
    assert abs(acc / n - want) < 0.045
    assert abs(scipy.stats.norm.cdf(-0.5) * 2 - 0.617) < 1e-3
    # the synthetic judge is a fair coin per slot
    assert abs(jacc / n - 0.5) < 0.05


# ----------------------------------------------------------------------------- top-K rule, plain-p resampling

def test_topk_rule_against_python_sort():
    # Sec. 5 "Training-free baseline": accept c iff it is among the K most probable target tokens.
    # Integer logits on a small vocabulary, with exact ties; rank by an independent Python sort.
    rng = np.random.default_rng(21)
    V, M, B = 6, 3, 40
    W = np.eye(V, dtype=np.float32)
    emb = rng.integers(-2, 3, size=(B, M + 1, V)).astype(np.float32)   # logits = emb rows (many ties)
    wj = np.zeros(V, dtype=np.float32)
    tokens = rng.integers(0, V, size=(B, M)).astype(np.int32)
    D = rng.normal(size=(B, M, V)).astype(np.float32)
    u = rng.random((B, M + 1)).astype(np.float32)
    prev = None
    for K in range(1, V + 1):
        out = vo.verify(emb, W, wj, tokens, D, u, mode=vo.MODE_STANDARD, rule=vo.RULE_TOPK, top_k=K)
        for b in range(B):
            zs = []
            for j in range(M):
                order = sorted(range(V), key=lambda v: (-float(emb[b, j, v]), v))  # ties: lower id first
                zs.append(int(order.index(int(tokens[b, j])) < K))
            assert out["z_stand"][b].tolist() == zs
            m = vo.accepted_prefix(zs)
            assert int(out["accept_len"][b]) == m
            row = [float(x) for x in emb[b, m]]
            assert int(out["next_token"][b]) == row.index(max(row))       # greedy target, lowest id on ties
        if prev is not None:                                              # acceptance is monotone in K
            assert (out["z_stand"] >= prev).all()
        prev = out["z_stand"].copy()
    # K = V: every draft token is accepted (the paper: "reduces to running just the fast draft model")
    assert (out["accept_len"] == M).all() and out["z_stand"].all()
    with pytest.raises(ValueError):
        vo.verify(emb, W, wj, tokens, D, u, rule=vo.RULE_TOPK, top_k=V + 1)


def test_top1_is_greedy_matching_and_judge_still_ors():
    shape = VerifyShape("t", 16, 6, 32, 200, "f32", 0.5)
    x = make_inputs(shape, 2)
    args = (x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"])
    L = vo.target_logits(x["emb"].reshape(-1, 32), x["W"]).reshape(16, 7, 200)
    out = vo.verify(*args, mode=vo.MODE_STANDARD, rule=vo.RULE_TOPK, top_k=1)
    greedy = (x["draft_tokens"] == np.argmax(L[:, :6], axis=-1))
    assert np.array_equal(out["z_stand"].astype(bool), greedy)            # Sec. 3.2: greedy matching
    assert greedy.any() and not greedy.all()
    jud = vo.verify(*args, mode=vo.MODE_JUDGE, rule=vo.RULE_TOPK, top_k=1)
    assert np.array_equal(jud["z_stand"], out["z_stand"]) and (jud["accept_len"] >= out["accept_len"]).all()
    # margins: distance to the top-K boundary is the logit gap to the best other token
    b, j = 0, 0
    c = int(x["draft_tokens"][b, j]); others = np.delete(L[b, j], c)
    assert abs(out["accept_margin"][b, j] - abs(L[b, j, c] - others.max())) < 1e-12
    srt = np.sort(L[b, int(out["accept_len"][b])])
    assert abs(out["sampler_margin"][b] - (srt[-1] - srt[-2])) < 1e-12


def test_resample_from_target_reading():
    # the literal reading of Sec. 3.1: after a rejection the token is drawn from p_i itself
    shape = VerifyShape("t", 24, 4, 16, 64, "f32", 2.0)
    x = make_inputs(shape, 5)
    args = (x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"])
    res = vo.verify(*args, mode=vo.MODE_STANDARD)
    tgt = vo.verify(*args, mode=vo.MODE_STANDARD, resample=vo.RESAMPLE_TARGET, return_probs=True)
    assert np.array_equal(res["accept_len"], tgt["accept_len"]) and np.array_equal(res["z_stand"], tgt["z_stand"])
    assert (tgt["accept_len"] < 4).any()
    for b in range(24):
        p = tgt["probs"][b, int(tgt["accept_len"][b])]
        want = int(np.searchsorted(np.cumsum(p), float(x["uniforms"][b, 4]) * p.sum(), side="right"))
        assert int(tgt["next_token"][b]) == want
    assert (res["next_token"] != tgt["next_token"]).any()
    assert (tgt["status"] == 0).all()


# ----------------------------------------------------------------------------- FP8 weights

def test_fp8_e4m3_decode_table():
    t = vo.E4M3FN
    # values fixed by the format: bias 7, 3 mantissa bits, no infinities, max 448
    known = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x38: 1.0, 0x3C: 1.5, 0x40: 2.0,
             0x7E: 448.0, 0xB8: -1.0, 0xFE: -448.0, 0x30: 0.5, 0x39: 1.125}
    for code, val in known.items():
        assert t[code] == val, hex(code)
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF]) and np.isfinite(t[:0x7F]).all()
    assert (np.diff(t[:0x7F]) > 0).all() and np.array_equal(t[0x80:0xFF], -t[0x00:0x7F])
    # independent library decode
    import torch
    ref = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.nan_to_num(ref, nan=-7.0), np.nan_to_num(t, nan=-7.0))
    # every finite code is exactly representable in bf16 (what the kernel converts to)
    f32 = t[np.isfinite(t)].astype(np.float32)
    assert np.array_equal(f32.view(np.uint32) & 0xFFFF, np.zeros(f32.size, dtype=np.uint32))


def test_fp8_weights_are_scaled_rows():
    from synth import CONFIGS
    shape = VerifyShape("t", 2, 4, 64, 300, "fp8", 1.0)
    x = make_inputs(shape, 1)
    assert x["W"].dtype == np.uint8 and x["w_scale"].shape == (300,) and x["emb"].dtype == np.uint16
    Weff = vo.E4M3FN[x["W"]] * x["w_scale"][:, None].astype(np.float64)
    X = vo.widen(x["emb"]).reshape(-1, 64)
    got = vo.target_logits(x["emb"].reshape(-1, 64), x["W"], w_scale=x["w_scale"])
    assert np.allclose(got, X @ Weff.T, rtol=1e-13, atol=1e-13)
    # quantisation error of the generator is what E4M3 allows: half a mantissa step at most
    out = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"],
                    w_scale=x["w_scale"])
    assert (out["status"] == 0).all()
    assert {"C2q", "C3q", "C4q"} <= set(CONFIGS)


# ----------------------------------------------------------------------------- INT8 weights

def test_int8_decode_is_twos_complement():
    # every bit pattern, decoded by the definition of two's complement: value = b - 256 * [b >= 128]
    pat = np.arange(256, dtype=np.uint8)
    got = vo.widen(pat.view(np.int8))
    assert got.dtype == np.float64
    assert [got[b] for b in (0x00, 0x01, 0x7F, 0x80, 0x81, 0xFF)] == [0.0, 1.0, 127.0, -128.0, -127.0, -1.0]
    assert np.array_equal(got, np.array([b - 256 * (b >= 128) for b in range(256)], dtype=np.float64))
    # every integer in [-128, 127] is exactly a bf16 value (what the kernel converts to)
    assert np.array_equal(got.astype(np.float32).view(np.uint32) & 0xFFFF, np.zeros(256, dtype=np.uint32))
    # same byte, other reading: the FP8 table must not be used for int8 arrays
    assert vo.widen(np.array([0x38], dtype=np.uint8))[0] == 1.0 and vo.widen(np.array([0x38], dtype=np.int8))[0] == 56.0


def test_int8_weights_are_scaled_rows():
    from synth import CONFIGS
    shape = VerifyShape("t", 2, 4, 64, 300, "int8", 1.0)
    x = make_inputs(shape, 1)
    assert x["W"].dtype == np.int8 and x["w_scale"].shape == (300,) and x["emb"].dtype == np.uint16
    # logits by hand for a few entries: integer weights, one scale per vocabulary entry
    X = vo.widen(x["emb"]).reshape(-1, 64)
    got = vo.target_logits(x["emb"].reshape(-1, 64), x["W"], temperature=2.0, w_scale=x["w_scale"])
    for r, v in ((0, 0), (3, 17), (9, 299)):
        want = sum(float(X[r, k]) * int(x["W"][v, k]) for k in range(64)) * float(x["w_scale"][v]) / 2.0
        assert abs(got[r, v] - want) <= 1e-12 * max(1.0, abs(want))
    # the [d, V] layout is the transpose
    got_t = vo.target_logits(x["emb"].reshape(-1, 64), np.ascontiguousarray(x["W"].T), temperature=2.0, w_layout="dv",
                             w_scale=x["w_scale"])
    assert np.array_equal(got, got_t)
    # the generator's quantisation: symmetric, full range used in every row, error at most half a step
    assert (np.abs(x["W"].astype(np.int32)).max(axis=1) == 127).all()
    out = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"],
                    w_scale=x["w_scale"])
    assert (out["status"] == 0).all()
    assert {"C2i", "C3i", "C4i"} <= set(CONFIGS)


# ----------------------------------------------------------------------------- pre-norm wiring (final RMS norm)

def test_round_to_bf16_hand_cases():
    # 8 significant bits, ties to even, written out by hand from the format
    cases = {
        1.0: 0x3F80,
        1.0 + 2.0 ** -8: 0x3F80,                 # exact tie between 1 and 1 + 2^-7: even mantissa wins
        1.0 + 2.0 ** -8 + 2.0 ** -40: 0x3F81,    # just above the tie
        1.0 + 2.0 ** -8 + 2.0 ** -30: 0x3F81,    # would round to the tie first if it went through float32
        1.0 + 3 * 2.0 ** -8: 0x3F82,             # tie between odd 0x3F81 and even 0x3F82
        -2.5: 0xC020, 0.0: 0x0000, 2.0 ** -133: 0x0001, 2.0 ** -134: 0x0000, 1.5 * 2.0 ** -133: 0x0002,
        3.3895313892515355e38: 0x7F7F, 3.4e38: 0x7F80,
    }
    xs = np.array(list(cases.keys()))
    assert [int(b) for b in vo.round_to_bf16_bits(xs)] == list(cases.values())
    assert int(vo.round_to_bf16_bits(np.array([-0.0]))[0]) == 0x8000
    # library conversion on float32-exact inputs (no double rounding possible there)
    import torch
    r = np.random.default_rng(3).standard_normal(200000).astype(np.float32) * np.float32(7.0)
    want = torch.from_numpy(r).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(vo.round_to_bf16_bits(r.astype(np.float64)), want)
    # rounding is idempotent and monotone
    b = vo.round_to_bf16_bits(r.astype(np.float64))
    assert np.array_equal(vo.round_to_bf16_bits(vo.widen(b)), b)
    srt = np.sort(r.astype(np.float64))
    assert (np.diff(vo.widen(vo.round_to_bf16_bits(srt))) >= 0).all()


def test_rmsnorm_definition():
    # hand case: h = (3, 4), gamma = (1, 2): mean square 12.5, x = (3, 8) / sqrt(12.5) = (0.848528.., 2.262741..)
    h = np.array([[3.0, 4.0]], dtype=np.float32); g = np.array([1.0, 2.0], dtype=np.float32)
    x, inv = vo.rmsnorm_rows(h, g, 0.0)
    assert x.dtype == np.float32 and abs(inv[0] - 1 / math.sqrt(12.5)) < 1e-15
    assert np.allclose(x, [[0.8485281374, 2.2627416998]], rtol=1e-7)
    xb, _ = vo.rmsnorm_rows(bf16_bits_from_f32(h), bf16_bits_from_f32(g), 0.0)
    assert xb.dtype == np.uint16 and [int(v) for v in xb[0]] == [0x3F59, 0x4011]   # 0.84765625, 2.265625
    # epsilon sits inside the square root, added to the MEAN square
    x, _ = vo.rmsnorm_rows(np.ones((1, 2), dtype=np.float32), np.ones(2, dtype=np.float32), 3.0)
    assert np.array_equal(x, [[0.5, 0.5]])
    # independent library routine, float64
    import torch
    rng = np.random.default_rng(0)
    h = (rng.standard_normal((5, 3, 96)) * rng.uniform(0.1, 30, size=(5, 3, 1))).astype(np.float32)
    g = (1 + 0.1 * rng.standard_normal(96)).astype(np.float32)
    want = torch.nn.functional.rms_norm(torch.from_numpy(h).double(), (96,), torch.from_numpy(g).double(), eps=1e-5).numpy()
    x32, inv = vo.rmsnorm_rows(h, g, 1e-5)
    assert np.array_equal(x32, want.astype(np.float32)) or np.allclose(x32, want, rtol=2e-7, atol=0)
    xb, _ = vo.rmsnorm_rows(bf16_bits_from_f32(h), bf16_bits_from_f32(g), 1e-5)
    hb = f32_from_bf16_bits(bf16_bits_from_f32(h)).astype(np.float64); gb = f32_from_bf16_bits(bf16_bits_from_f32(g)).astype(np.float64)
    wantb = torch.nn.functional.rms_norm(torch.from_numpy(hb), (96,), torch.from_numpy(gb), eps=1e-5).numpy()
    got = vo.widen(xb)
    assert (np.abs(got - wantb) <= np.abs(wantb) * 2.0 ** -8 + 1e-300).all()          # within half a bf16 step
    assert (np.abs(got - wantb) <= np.abs(vo.widen(xb + 1) - wantb) + 1e-300).all()     # and nearer than the next code
    # invariants: unit gain, eps = 0 -> unit rms; scaling a row by a power of two changes nothing at all
    x1, _ = vo.rmsnorm_rows(h, np.ones(96, dtype=np.float32), 0.0)
    assert np.allclose(np.sqrt(np.mean(x1.astype(np.float64) ** 2, axis=-1)), 1.0, atol=1e-6)
    x2, _ = vo.rmsnorm_rows(bf16_bits_from_f32(h * 4), bf16_bits_from_f32(g), 0.0)
    x3, _ = vo.rmsnorm_rows(bf16_bits_from_f32(h), bf16_bits_from_f32(g), 0.0)
    assert np.array_equal(x2, x3)


def test_prenorm_wiring_of_the_judge():
    # Sec. 4.1: LM head after the final RMS norm, judge on the embedding before it
    from synth import RMS_EPS
    shape = VerifyShape("t", 6, 5, 64, 200, "bf16", 1.0)
    x = make_inputs(shape, 4, prenorm=True)
    assert "emb" not in x and x["hidden"].dtype == np.uint16 and x["gamma"].shape == (64,) and x["rms_eps"] == RMS_EPS
    emb, inv = vo.rmsnorm_rows(x["hidden"], x["gamma"], x["rms_eps"])
    out = vo.verify(emb, x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"],
                    emb_judge=x["hidden"], return_probs=True)
    H = vo.widen(x["hidden"]); w = vo.widen(x["w_judge"])
    assert np.allclose(out["judge_logit"], np.einsum("bjk,k->bj", H[:, 1:, :], w), rtol=1e-13, atol=1e-13)
    # the LM head saw the normalised rows: probabilities are those of softmax(norm(h) W)
    Xn = vo.widen(emb).reshape(-1, 64)
    L = (Xn @ vo.widen(x["W"]).T)
    P = np.exp(L - L.max(1, keepdims=True)); P /= P.sum(1, keepdims=True)
    assert np.allclose(out["probs"].reshape(-1, 200), P, rtol=1e-12, atol=1e-15)
    # rows have very different scales before the norm and unit-ish rms after it
    rms_before = np.sqrt(np.mean(H ** 2, axis=-1)); rms_after = np.sqrt(np.mean(vo.widen(emb) ** 2, axis=-1))
    assert rms_before.max() / rms_before.min() > 3 and np.allclose(rms_after, 1.0, atol=0.1)
    # with delta = 0.5 and no bias the judge decision is the sign of w.h, which the positive row
    # scale 1/rms cannot change: judging the scaled row gives the same mask
    scaled = (H * inv[..., None])
    assert np.array_equal(out["z_judge"], (np.einsum("bjk,k->bj", scaled[:, 1:, :], w) > 0).astype(out["z_judge"].dtype))
    # a sane workload: the draft is a noisy copy of the target, so some but not all slots pass
    assert 0 < out["z_stand"].mean() < 1 and (out["status"] == 0).all()


# ----------------------------------------------------------------------------- the step after: growing the context

def test_append_tokens_hand_cases():
    # Sec. 3.1: accepted tokens, then the one new token, are added to the context
    buf = np.full((3, 6), -1, dtype=np.int32); buf[0, 0] = 7
    lengths = np.array([1, 0, 5], dtype=np.int64)
    draft = np.array([[5, 6, 9], [1, 2, 3], [11, 12, 13]], dtype=np.int32)
    vo.append_tokens(buf, lengths, draft, np.array([2, 0, 3]), np.array([8, 4, 14]))
    assert buf[0].tolist() == [7, 5, 6, 8, -1, -1] and lengths[0] == 4      # two accepted + replacement
    assert buf[1].tolist() == [4, -1, -1, -1, -1, -1] and lengths[1] == 1   # nothing accepted: only the new token
    assert buf[2].tolist() == [-1, -1, -1, -1, -1, 11] and lengths[2] == 6  # full buffer: the rest is dropped
    vo.append_tokens(buf, lengths, draft, np.array([3, 3, 3]), np.array([8, 4, 14]))
    assert buf[0].tolist() == [7, 5, 6, 8, 5, 6] and lengths[0] == 6 and lengths[2] == 6
    assert buf[1].tolist() == [4, 1, 2, 3, 4, -1] and lengths[1] == 5
    # a call always emits accept_len + 1 tokens: at least one, at most M + 1
    x = make_inputs(VerifyShape("t", 16, 4, 16, 64, "f32", 1.5), 2)
    out = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"])
    buf = np.zeros((16, 8), dtype=np.int32); lengths = np.zeros(16, dtype=np.int64)
    vo.append_tokens(buf, lengths, x["draft_tokens"], out["accept_len"], out["next_token"])
    assert np.array_equal(lengths, out["accept_len"] + 1) and lengths.min() >= 1 and lengths.max() <= 5
    for b in range(16):
        n = int(out["accept_len"][b])
        assert np.array_equal(buf[b, :n], x["draft_tokens"][b, :n]) and buf[b, n] == out["next_token"][b]


def test_masked_draft_tokens_and_rows():
    # a filtered draft: -inf logits have probability zero; a drafted token with q[c] = 0 passes Eq. 4
    # iff p[c] > 0 (the division-free form eps * 0 < p); a row of nothing but -inf is no distribution
    x = make_inputs(VerifyShape("t", 2, 3, 16, 40, "f32", 1.0), 3)
    D = x["draft_logits"].copy()
    c = int(x["draft_tokens"][0, 1])
    D[0, 1, c] = -np.inf
    D[0, 0, :10] = -np.inf
    with np.errstate(invalid="ignore"):
        out = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], D, x["uniforms"], mode=vo.MODE_STANDARD)
    assert out["q_at_draft"][0, 1] == 0.0 and out["z_stand"][0, 1] == 1 and (out["status"] == 0).all()
    q0 = scipy.special.softmax(D[0, 0].astype(np.float64))
    assert (q0[:10] == 0).all() and abs(out["q_at_draft"][0, 0] - q0[int(x["draft_tokens"][0, 0])]) < 1e-15
    D[1, 2, :] = -np.inf
    with np.errstate(invalid="ignore"):
        out = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], D, x["uniforms"], mode=vo.MODE_STANDARD)
    assert out["status"].tolist() == [0, vo.STATUS_NAN]


# ----------------------------------------------------------------------------- metamorphic relations

def _verify(x, **kw):
    return vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"], **kw)


def test_sequences_are_independent_and_order_free():
    # no step of the method crosses sequences (Sec. 3.1: each context is verified on its own)
    x = make_inputs(VerifyShape("t", 7, 5, 32, 96, "f32", 1.2), 8)
    out = _verify(x)
    perm = np.array([3, 0, 6, 1, 5, 2, 4])
    y = dict(x)
    for k in ("emb", "draft_tokens", "draft_logits", "uniforms"):
        y[k] = x[k][perm]
    outp = _verify(y)
    for k, v in out.items():
        assert np.array_equal(outp[k], v[perm], equal_nan=True), k


def test_vocabulary_relabelling():
    # renaming the tokens (rows of W_lm, columns of the draft, drafted ids) changes no decision;
    # the new token is the renamed old one whenever the CDF order plays no role (everything accepted
    # is not such a case, so only the masks and the prefix are compared)
    x = make_inputs(VerifyShape("t", 9, 6, 32, 80, "f32", 1.0), 12)
    out = _verify(x)
    pi = np.random.default_rng(0).permutation(80)          # new id of old token v is inv[v]
    inv = np.empty(80, dtype=np.int64); inv[pi] = np.arange(80)
    y = dict(x)
    y["W"] = x["W"][pi]                                    # row new_id holds old token pi[new_id]
    y["draft_logits"] = x["draft_logits"][:, :, pi]
    y["draft_tokens"] = inv[x["draft_tokens"]].astype(np.int32)
    outp = _verify(y)
    away = (out["accept_margin"] > 1e-9) & (out["judge_margin"] > 1e-9)
    assert away.all()
    for k in ("z_stand", "z_judge", "accept_len"):
        assert np.array_equal(out[k], outp[k]), k
    assert np.allclose(out["p_at_draft"], outp["p_at_draft"], rtol=1e-12) and np.allclose(out["q_at_draft"], outp["q_at_draft"], rtol=1e-12)


def test_draft_logit_shift_and_truncated_drafts():
    x = make_inputs(VerifyShape("t", 8, 6, 32, 96, "f32", 1.5), 14)
    out = _verify(x)
    # softmax is shift invariant: a constant added to a draft row changes nothing away from ties
    y = dict(x); y["draft_logits"] = (x["draft_logits"].astype(np.float64) + 3.25).astype(np.float32)
    outs = _verify(y)
    assert (out["accept_margin"] > 1e-6).all() and (out["sampler_margin"] > 1e-6).all()
    for k in ("z_stand", "z_judge", "accept_len", "next_token"):
        assert np.array_equal(out[k], outs[k]), k
    # verifying only the first M' drafted tokens: same masks on those slots, prefix cut at M', and the same
    # new token whenever the cut fell before M' (same row, same residual, same sampler draw)
    Mp = 3
    z = dict(x)
    z["emb"] = x["emb"][:, :Mp + 1]; z["draft_tokens"] = x["draft_tokens"][:, :Mp]
    z["draft_logits"] = x["draft_logits"][:, :Mp + 1]
    z["uniforms"] = np.concatenate([x["uniforms"][:, :Mp], x["uniforms"][:, 6:7]], axis=1)
    outt = _verify(z)
    assert np.array_equal(outt["z_stand"], out["z_stand"][:, :Mp]) and np.array_equal(outt["z_judge"], out["z_judge"][:, :Mp])
    assert np.array_equal(outt["accept_len"], np.minimum(out["accept_len"], Mp))
    early = out["accept_len"] < Mp
    assert early.any() and np.array_equal(outt["next_token"][early], out["next_token"][early])


# ----------------------------------------------------------------------------- the comparison itself

def test_comparison_accepts_the_oracle_and_catches_planted_mistakes():
    from oracle.compare import compare
    shape = VerifyShape("t", 4, 6, 64, 300, "bf16", 1.0)
    x = make_inputs(shape, 2)
    ref = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"], return_probs=True)

    def as_library(r):   # the output types of the library
        o = {k: np.array(v) for k, v in r.items()}
        for k in ("p_at_draft", "q_at_draft", "judge_logit", "row_max", "row_sumexp", "probs"):
            o[k] = o[k].astype(np.float32)
        return o

    compare(as_library(ref), ref)

    def planted(mutate):
        g = as_library(ref)
        mutate(g)
        with pytest.raises(AssertionError):
            compare(g, ref)

    b = int(np.argmax(ref["accept_len"] < 6))                          # a sequence with a rejection
    planted(lambda g: g["accept_len"].__setitem__(b, g["accept_len"][b] + 1))
    planted(lambda g: g["next_token"].__setitem__(0, (g["next_token"][0] + 7) % 300))
    planted(lambda g: g["p_at_draft"].__setitem__((0, 0), g["p_at_draft"][0, 0] * 1.01))
    planted(lambda g: g["q_at_draft"].__setitem__((1, 2), g["q_at_draft"][1, 2] * 0.99))
    planted(lambda g: g["judge_logit"].__setitem__((2, 1), g["judge_logit"][2, 1] + 0.01))
    planted(lambda g: g["status"].__setitem__(3, 2))
    planted(lambda g: g["probs"].__setitem__((0, 0, 5), g["probs"][0, 0, 5] * 1.01))
    j = int(ref["accept_len"][b])                                       # flip the rejecting slot's standard bit
    if ref["accept_margin"][b, j] >= 1e-5 and not ref["z_judge"][b, j]:
        planted(lambda g: g["z_stand"].__setitem__((b, j), 1))
    # values below float32's normal range: the library may return anything that small, nothing larger
    tiny = {k: np.array(v) for k, v in ref.items()}
    tiny["p_at_draft"] = tiny["p_at_draft"].copy(); tiny["p_at_draft"][0, 0] = 1e-60
    g = as_library(tiny); assert g["p_at_draft"][0, 0] == 0.0
    compare(g, tiny)
    g["p_at_draft"][0, 0] = 1e-30
    with pytest.raises(AssertionError):
        compare(g, tiny)


# ----------------------------------------------------------------------------- the helpers that decide what parity may excuse

def _py_first_over(mass, thresh):
    """Ascending-id scan with a running sum (the order numpy's cumsum uses): first token whose cumulative
    mass exceeds thresh, else the last token with mass."""
    run, last = 0.0, -1
    for v, x in enumerate(mass):
        run += float(x)
        if x > 0:
            last = v
        if run > thresh:
            return v
    return last


def test_mass_neighbours_against_a_scan():
    # zero runs at both ends and in the middle, single-token support, empty support
    cases = [
        [0, 0, 3, 0, 0, 1, 2, 0, 0, 0, 5, 0, 0],
        [1, 0, 0, 0, 0, 0, 0, 1],
        [0, 0, 0, 4, 0, 0],
        [2, 3, 4],
        [0, 0, 0],
    ]
    rng = np.random.default_rng(31)
    for _ in range(30):
        cases.append((rng.random(40) * (rng.random(40) > 0.6)).tolist())
    for mass in cases:
        mass = np.asarray(mass, dtype=np.float64)
        for v in range(len(mass)):
            below = -1
            for t in range(v - 1, -1, -1):
                if mass[t] > 0:
                    below = t
                    break
            above = -1
            for t in range(v + 1, len(mass)):
                if mass[t] > 0:
                    above = t
                    break
            assert vo.mass_neighbours(mass, v) == (below, above), (mass, v)
    # the neighbour is NOT simply the adjacent id
    assert vo.mass_neighbours(np.array([1.0, 0.0, 0.0, 2.0, 0.0, 3.0]), 3) == (0, 5)


def test_inverse_cdf_margin_is_the_distance_to_the_nearest_edge():
    # Moving the threshold by just more than margin * S towards the nearer edge changes the token, to the
    # neighbour that carries mass on that side; by just less, in either direction, it does not.
    rng = np.random.default_rng(32)
    moved_up = moved_down = 0
    for trial in range(300):
        V = int(rng.integers(3, 60))
        mass = rng.random(V) * (rng.random(V) > 0.4)
        if not (mass > 0).any():
            continue
        S = float(np.sum(mass))
        u = float(rng.random())
        tok, margin = vo.inverse_cdf(mass, u)
        thresh = u * S
        assert tok == _py_first_over(mass, thresh)
        below, above = vo.mass_neighbours(mass, tok)
        if margin < 1e-6:
            continue
        step_in, step_out = margin * S * (1 - 1e-6), margin * S * (1 + 1e-6)
        first = lambda t: _py_first_over(mass, t) if t >= 0 else tok   # a threshold u * S is never negative
        assert first(thresh + step_in) == tok and first(thresh - step_in) == tok
        up, down = first(thresh + step_out), first(thresh - step_out)
        if up == tok and down == tok:
            # only possible for the last token with mass when its upper edge (the total mass, which no u < 1
            # reaches) is the nearer one: the margin then understates, never overstates, the room
            run = 0.0
            for t in mass:
                run += float(t)
            assert above < 0 and thresh + step_out >= run * (1 - 1e-12), "margin overstates the distance to both edges"
        if up != tok:
            assert up == above, (mass, u, tok, up, above)   # for the last token with mass the scan falls back to it
            moved_up += 1
        if down != tok:
            assert down == below and below >= 0
            moved_down += 1
        if below < 0:   # nothing below carries mass: only the upper edge counts
            assert down == tok
            cum = float(np.cumsum(mass)[tok])
            assert abs(margin - (cum - thresh) / S) < 1e-15
    assert moved_up > 30 and moved_down > 30
    # hand case: mass 1, 0, 2, 1 (S = 4), u = 0.3: threshold 1.2 lies 0.2 above the edge at 1 and 1.8 below the edge at 3
    tok, margin = vo.inverse_cdf(np.array([1.0, 0.0, 2.0, 1.0]), 0.3)
    assert tok == 2 and abs(margin - 0.2 / 4) < 1e-15
    # the last token with mass has no upper neighbour: crossing its upper edge is impossible (u < 1)
    tok, margin = vo.inverse_cdf(np.array([1.0, 3.0, 0.0]), 0.9)
    assert tok == 1 and abs(margin - 0.1) < 1e-12 and vo.mass_neighbours(np.array([1.0, 3.0, 0.0]), 1) == (0, -1)


def _py_rank(row, c):
    order = sorted(range(len(row)), key=lambda v: (-float(row[v]), v))   # ties: lower id first
    return order.index(c)


def test_topk_margin_for_every_k_with_ties():
    # Quarter-integer logits: many exact ties, exact float64 arithmetic.  Shifting L[c] by just more than the
    # margin across the boundary flips "c is among the top K", by just less it does not.
    rng = np.random.default_rng(33)
    flips = 0
    for trial in range(60):
        V = int(rng.integers(2, 12))
        row = rng.integers(-6, 7, size=V).astype(np.float64) / 4.0
        for c in range(V):
            for K in range(1, V + 1):
                accepted = _py_rank(row, c) < K
                assert (vo.rank_of(row, c) < K) == accepted
                mg = vo.topk_margin(row, c, K)
                assert mg >= 0
                if K == V:
                    assert accepted and mg == math.inf   # nothing can push c out of the top V
                    continue
                sign = -1.0 if accepted else 1.0         # direction that crosses the boundary
                over, under = row.copy(), row.copy()
                over[c] += sign * (mg + 1e-9)
                assert (_py_rank(over, c) < K) != accepted, (row, c, K, mg)
                flips += 1
                if mg > 1e-9:
                    under[c] += sign * (mg - 1e-9)
                    assert (_py_rank(under, c) < K) == accepted, (row, c, K, mg)
                else:
                    # margin 0 = an exact tie at the boundary, decided by the token ids
                    others = sorted((float(x) for i, x in enumerate(row) if i != c), reverse=True)
                    assert others[K - 1] == row[c]
    assert flips > 1000
    # hand case: logits 5, 3, 3, 1, K = 2: token 1 (3.0, wins the tie by id) is in, token 2 is out, both by margin 0;
    # token 0 is in by 2 (the 2nd largest other is 3), token 3 is out by 2
    row = np.array([5.0, 3.0, 3.0, 1.0])
    assert [vo.topk_margin(row, c, 2) for c in range(4)] == [2.0, 0.0, 0.0, 2.0]
    assert [vo.rank_of(row, c) < 2 for c in range(4)] == [True, True, False, False]


def test_new_token_for_a_given_prefix():
    # new_token_for_prefix(b, m) is step 7 with the prefix forced to m: equal to verify()'s token at verify()'s own
    # prefix, and equal to a scalar evaluation of the definition at every other prefix
    shape = VerifyShape("t", 12, 5, 32, 90, "f32", 1.5)
    x = make_inputs(shape, 3)
    args = (x["emb"], x["W"], x["draft_logits"], x["uniforms"])
    out = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"])
    assert len(set(out["accept_len"].tolist())) >= 3
    Wd = x["W"].astype(np.float64)
    for b in range(shape.B):
        tok, margin, lo, hi = vo.new_token_for_prefix(*args, b, int(out["accept_len"][b]))
        assert (tok, lo, hi) == (int(out["next_token"][b]), int(out["next_below"][b]), int(out["next_above"][b]))
        assert abs(margin - out["sampler_margin"][b]) < 1e-12      # a one-row product may sum in another order
        for m in range(shape.M + 1):
            p = py_softmax([float(np.dot(x["emb"][b, m].astype(np.float64), Wd[v])) for v in range(shape.V)])
            if m < shape.M:
                q = py_softmax([float(t) for t in x["draft_logits"][b, m]])
                mass = [max(0.0, pv - qv) for pv, qv in zip(p, q)]
            else:
                mass = p
            S = 0.0
            for t in mass:
                S += t
            want = _py_first_over(mass, float(x["uniforms"][b, shape.M]) * S)
            got = vo.new_token_for_prefix(*args, b, m)
            assert got[0] == want or got[1] < 1e-12, (b, m)
    # plain-p replacement and the greedy rule go through the same wrapper
    t_res = vo.new_token_for_prefix(*args, 0, 0)[0]
    t_tgt = vo.new_token_for_prefix(*args, 0, 0, resample=vo.RESAMPLE_TARGET)[0]
    ref_tgt = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"],
                        resample=vo.RESAMPLE_TARGET, seqs=[0])
    if int(ref_tgt["accept_len"][0]) == 0:
        assert t_tgt == int(ref_tgt["next_token"][0])
    L0 = vo.target_logits(x["emb"][0, 2:3], x["W"])[0]
    assert vo.new_token_for_prefix(*args, 0, 2, rule=vo.RULE_TOPK)[0] == int(np.argmax(L0))
    assert isinstance(t_res, int)
    with pytest.raises(ValueError):
        vo.new_token_for_prefix(*args, 0, shape.M + 1)


def _library_types(r):
    o = {k: np.array(v) for k, v in r.items()}
    for k in ("p_at_draft", "q_at_draft", "judge_logit", "row_max", "row_sumexp"):
        o[k] = o[k].astype(np.float32)
    return o


def test_comparison_bands_have_the_stated_widths():
    # A flipped mask bit is excused only inside the stated band (|p/q - eps| < 1e-5; judge logit within 1e-4 of
    # its threshold), a different new token only inside the sampler band (1e-5 of the total mass) AND only for
    # the neighbouring token that carries mass.
    from oracle.compare import compare
    V, M = 8, 2
    P0 = [.2, .05, .3, .35, .02, .03, .03, .02]
    Q0 = [.1, .15, .1, .05, .12, .13, .2, .15]      # residual of row 0: .1, 0, .2, .3, 0, 0, 0, 0 (S = .6)
    P1 = [.25] + [.75 / 7] * 7
    Q1 = [.5] + [.5 / 7] * 7                          # token 0 at slot 1: p/q = 0.5
    P2 = [.125] * 8
    P, Q = np.array([P0, P1, P2]), np.array([Q0, Q1])

    def case(tokens, jbits, u, **kw):
        return direct_case(P, Q, jbits, tokens, u, **kw)

    def flipped(ref, key, idx):
        g = _library_types(ref)
        g[key][idx] = 1 - g[key][idx]
        z = g["z_stand"].astype(bool) | g["z_judge"].astype(bool)
        g["accept_len"][0] = int(np.argmin(np.append(z[0], False)))
        return g

    # --- standard test, slot 1: ratio 0.5, u = 0.5 + 2e-5 is outside the band, 0.5 + 5e-6 inside
    far = case([[2, 0]], [1, 0], [0.3, 0.5 + 2e-5, 0.7])
    near = case([[2, 0]], [1, 0], [0.3, 0.5 + 5e-6, 0.7])
    assert not far["z_stand"][0, 1] and not near["z_stand"][0, 1]
    assert 1.9e-5 < far["accept_margin"][0, 1] < 2.1e-5 and 4e-6 < near["accept_margin"][0, 1] < 6e-6
    with pytest.raises(AssertionError):
        compare(flipped(far, "z_stand", (0, 1)), far)
    rep = compare(flipped(near, "z_stand", (0, 1)), near)
    assert rep["near_tie_stand"] == 1 and rep["excluded_sequences"] == 1
    # --- judge test, slot 1: logit = 1 + bias against threshold 0
    farj = case([[2, 0]], [1, 1], [0.3, 0.9, 0.7], judge_bias=-1.0 + 2e-4)
    nearj = case([[2, 0]], [1, 1], [0.3, 0.9, 0.7], judge_bias=-1.0 + 5e-5)
    assert farj["z_judge"][0, 1] and nearj["z_judge"][0, 1] and not farj["z_stand"][0, 1]
    assert 1.9e-4 < farj["judge_margin"][0, 1] < 2.1e-4 and 4e-5 < nearj["judge_margin"][0, 1] < 6e-5
    with pytest.raises(AssertionError):
        compare(flipped(farj, "z_judge", (0, 1)), farj)
    rep = compare(flipped(nearj, "z_judge", (0, 1)), nearj)
    assert rep["near_tie_judge"] == 1 and rep["excluded_sequences"] == 1
    # slot 0 of the same cases is decided far from its threshold (logit -1 + bias): never excused
    with pytest.raises(AssertionError):
        compare(flipped(nearj, "z_stand", (0, 0)), nearj)
    # --- sampler: reject slot 0 (token 1: p/q = 1/3, u = 0.9, judge says no); residual CDF edges .1 .1 .3 .6
    s_near = case([[1, 0]], [0, 0], [0.9, 0.5, 0.5 + 5e-6])      # threshold 5e-6 * S above the edge at .3
    s_far = case([[1, 0]], [0, 0], [0.9, 0.5, 0.5 + 2e-5])
    for r in (s_near, s_far):
        assert int(r["accept_len"][0]) == 0 and int(r["next_token"][0]) == 3
        assert (int(r["next_below"][0]), int(r["next_above"][0])) == (2, -1)
    assert 4e-6 < s_near["sampler_margin"][0] < 6e-6 and 1.9e-5 < s_far["sampler_margin"][0] < 2.1e-5

    def with_token(ref, tok):
        g = _library_types(ref)
        g["next_token"][0] = tok
        return g

    assert compare(with_token(s_near, 2), s_near)["near_tie_sampler"] == 1   # the neighbour with mass, inside the band
    for tok in (1, 0, 4, 7):   # the adjacent id without mass, a token two edges away, tokens above
        with pytest.raises(AssertionError):
            compare(with_token(s_near, tok), s_near)
    with pytest.raises(AssertionError):   # the same neighbour, outside the band
        compare(with_token(s_far, 2), s_far)
    # --- a flipped bit inside the band moves the prefix: with replay the token is held to that prefix
    g = flipped(near, "z_stand", (0, 1))            # library accepts slot 1 too: prefix 2, bonus token from P2
    assert int(g["accept_len"][0]) == 2 and int(near["accept_len"][0]) == 1
    emb = np.log(P).astype(np.float32)[None]
    Qd = np.concatenate([Q, np.zeros((1, V))]).astype(np.float32)[None]
    unif = np.array([[0.3, 0.5 + 5e-6, 0.7]], dtype=np.float32)

    def replay(b, m):
        return vo.new_token_for_prefix(emb, np.eye(V, dtype=np.float32), Qd, unif, b, m, draft_kind=vo.DRAFT_PROBS)

    want = replay(0, 2)[0]
    assert want == 5                                # uniform P2, u_s = 0.7 -> floor(0.7 * 8)
    g["next_token"][0] = want
    rep = compare(g, near, replay=replay)
    assert rep["replayed_sequences"] == 1 and rep["excluded_sequences"] == 1
    g["next_token"][0] = int(near["next_token"][0]) if int(near["next_token"][0]) != want else 0
    compare(g, near)                                # without replay the token of an excluded sequence is not looked at
    with pytest.raises(AssertionError):
        compare(g, near, replay=replay)
