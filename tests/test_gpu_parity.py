"""GPU parity: the HIP library against the float64 oracle, element by element, on the
same seeded inputs.  Every case goes through the C ABI (ctypes binding)."""

import numpy as np
import pytest

from oracle import verify_oracle as vo
from oracle.compare import compare as _compare
from synth import CONFIGS, VerifyShape, bf16_bits_from_f32, make_inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def jd():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a HIP device"
    from paper_2501_19309_amd import binding, harness
    binding.load_library()
    return harness


class Ref(dict):
    """The oracle's outputs plus ``replay(b, m)``: its step 7 for row b of these outputs under a forced prefix m."""
    replay = None


def abi_floats(kw):
    # delta, judge_bias and temperature cross the C ABI as float32: the oracle gets the values the library gets
    for k in ("delta", "judge_bias", "temperature"):
        if k in kw:
            kw[k] = float(np.float32(kw[k]))
    return kw


def oracle_call(emb, x, draft=None, **kw):
    kw = abi_floats(dict(kw))
    if "w_scale" in x:
        kw.setdefault("w_scale", x["w_scale"])
    draft = x["draft_logits"] if draft is None else draft
    ref = Ref(vo.verify(emb, x["W"], x["w_judge"], x["draft_tokens"], draft, x["uniforms"], **kw))
    rows = list(range(emb.shape[0])) if kw.get("seqs") is None else [int(b) for b in kw["seqs"]]
    step7 = {k: kw[k] for k in ("draft_kind", "temperature", "w_layout", "rule", "resample", "w_scale") if k in kw}
    ref.replay = lambda b, m: vo.new_token_for_prefix(emb, x["W"], draft, x["uniforms"], rows[b], m, **step7)
    return ref


def oracle_for(x, **kw):
    return oracle_call(x["emb"], x, **kw)


def compare(got, ref, **kw):
    """The parity bar of oracle/compare.py; where a near-tie moved the library's prefix, its token is held to the
    oracle's step 7 for that prefix (refs built by oracle_call carry the replay)."""
    return _compare(got, ref, replay=getattr(ref, "replay", None), **kw)


SMALL = [
    # name, B, M, d, V, dtype, noise  -- several vocabulary groups / K chunks and ragged tails
    VerifyShape("s_f32_tiny", 1, 5, 256, 1024, "f32", 1.0),
    VerifyShape("s_f32_ragged", 3, 7, 100, 1000, "f32", 1.5),
    VerifyShape("s_bf16_1blk", 1, 5, 256, 1024, "bf16", 1.0),
    VerifyShape("s_bf16_2blk", 1, 25, 512, 2048, "bf16", 1.0),
    VerifyShape("s_bf16_ragged", 2, 9, 264, 1000, "bf16", 2.0),     # d % 256 != 0, V % 64 != 0, R = 20
    VerifyShape("s_bf16_3blk", 3, 12, 320, 4100, "bf16", 1.0),      # R = 39
    VerifyShape("s_bf16_4blk", 4, 15, 768, 3000, "bf16", 1.5),      # R = 64
    VerifyShape("s_bf16_batched", 9, 10, 512, 5000, "bf16", (0.5, 2.5)),  # R = 99 > 64
]


EDGE = [
    VerifyShape("e_M63", 2, 63, 64, 300, "bf16", 1.0),          # ballot width: M = 63, R = 128 (GEMM regime)
    VerifyShape("e_M63_single", 1, 63, 128, 512, "bf16", 1.5),   # R = 64 exactly (largest small-row launch)
    VerifyShape("e_M1", 5, 1, 64, 200, "bf16", 1.0),             # one draft token
    VerifyShape("e_V8_f32", 7, 3, 16, 8, "f32", 1.0),            # vocabulary of 8 (brute-force scale)
    VerifyShape("e_V8_bf16", 7, 3, 16, 8, "bf16", 1.0),          # one partial vocabulary group
    VerifyShape("e_V65", 3, 4, 32, 65, "bf16", 0.5),             # one entry into the second group
    VerifyShape("e_d8", 2, 5, 8, 700, "bf16", 1.0),              # smallest hidden size the bf16 path takes
    VerifyShape("e_B200", 200, 2, 64, 333, "bf16", 1.0),         # many sequences, R = 600
    VerifyShape("e_R65", 5, 12, 96, 1024, "bf16", 1.0),          # first row count of the GEMM regime
    VerifyShape("e_R177", 3, 58, 64, 640, "bf16", 1.0),          # first row count of the 352-row kernel (6 row blocks per half)
    VerifyShape("e_R352", 32, 10, 520, 4100, "bf16", (0.5, 2.0)),  # exactly one 352-row tile, 24 K steps, ragged V
    VerifyShape("e_R400", 40, 9, 264, 1000, "bf16", 1.0),        # two equally sized row tiles of the 352-row kernel
    VerifyShape("e_R1000", 100, 9, 128, 700, "bf16", 1.0),       # three full 352-row tiles, the last one ragged
    VerifyShape("e_R704_M63", 11, 63, 72, 130, "bf16", 1.0),     # two full 352-row tiles, widest ballot, 3 vocabulary groups
    VerifyShape("e_R352_d8", 44, 7, 8, 300, "bf16", 1.0),        # 352-row tiling at the smallest hidden size (one real K step)
    VerifyShape("e_R300_V9", 30, 9, 40, 9, "bf16", 1.0),         # 352-row tiling with one partial vocabulary group
    VerifyShape("e_V1", 2, 2, 8, 1, "f32", 1.0),                 # single token vocabulary: everything is certain
    VerifyShape("e_R2816", 256, 10, 256, 3000, "bf16", (0.5, 2.0)),  # eight 352-row tiles: several rounds of workgroups per unit
    VerifyShape("e_R2640_fp8", 240, 10, 272, 1500, "fp8", (0.5, 2.0)),  # eight row tiles of 330 rows, FP8 codes, ragged d
    VerifyShape("e_B70000", 70000, 1, 16, 40, "bf16", 1.0),      # more sequences (and rows) than a grid's y dimension holds
    VerifyShape("e_R264", 24, 10, 264, 2100, "bf16", (0.5, 2.0)),  # 264 rows: a 352-row tile three quarters full
    VerifyShape("e_R528", 48, 10, 264, 2100, "bf16", (0.5, 2.0)),  # 528 rows: two row tiles of 264 rows
]


@pytest.mark.parametrize("shape", EDGE, ids=lambda s: s.name)
def test_edge_shapes_match_oracle(jd, shape):
    print(f"[case] {shape.name}", flush=True)
    x = make_inputs(shape, 4)
    ref = oracle_for(x, return_probs=True)
    got = jd.run_once(x, want_probs=True)
    rep = compare(got, ref)
    print(rep, flush=True)


@pytest.mark.parametrize("shape", SMALL, ids=lambda s: s.name)
@pytest.mark.parametrize("seed", [0, 1])
def test_small_shapes_match_oracle(jd, shape, seed):
    print(f"[case] {shape.name} seed={seed}", flush=True)
    x = make_inputs(shape, seed)
    ref = oracle_for(x, return_probs=True)
    got = jd.run_once(x, want_probs=True)
    rep = compare(got, ref)
    print(rep, flush=True)


@pytest.mark.parametrize("dtype", ["bf16", "fp8", "int8"])
def test_row_block_counts_of_the_176_row_kernel(jd, dtype):
    # The 176-row kernel (65 .. 176 rows) is instantiated per number of 16-row blocks that hold rows (5 .. 11): one
    # shape per instantiation, the last block ragged, and the exact block boundaries 80 and 176.
    seen = set()
    for B, M in [(7, 10), (13, 6), (9, 11), (25, 4), (14, 9), (31, 4), (12, 13), (5, 15), (16, 10)]:
        R = B * (M + 1)
        assert 64 < R <= 176, R
        live = (R + 15) // 16
        seen.add(live)
        shape = VerifyShape(f"live_{dtype}_R{R}", B, M, 144, 600, dtype, 1.2)
        print(f"[case] {shape.name} ({live} row blocks)", flush=True)
        x = make_inputs(shape, 11)
        compare(jd.run_once(x), oracle_for(x))
    assert seen == set(range(5, 12)), seen


@pytest.mark.parametrize("dtype", ["bf16", "fp8", "int8"])
def test_row_tiles_of_the_352_row_kernel(jd, dtype):
    # Above 176 rows the 352-row kernel cuts a call into row tiles of two halves with 6 .. 11 sixteen-row blocks each
    # (one instantiation per block count): one tile sized to its rows; several equally sized tiles if they need at
    # most 9 blocks per half; else full tiles with the last one in a launch of its own if that needs at most 8 blocks
    # per half; else equal tiles of 10 blocks per half or full tiles.  Every instantiation in every form, rows ending inside half 0, at its end, inside half 1, and a single
    # row in the last tile.
    def plan(R):
        tiles = -(-R // 352)
        if tiles == 1:
            return "one", max(6, -(-R // 32)), None
        nb = -(-R // (32 * tiles))
        if nb <= 9:
            return "equal", nb, None
        last = max(6, -(-(R - (tiles - 1) * 352) // 32))
        if last <= 8:
            return "full", 11, last
        return ("equal", 10, None) if nb == 10 else ("full", 11, 11)
    cases = [(3, 58), (20, 9), (24, 9), (27, 9), (30, 9), (34, 9),          # 177 .. 340 rows: one tile, 6 .. 11 blocks per half
             (12, 15), (13, 15), (18, 15), (22, 15),                        # 192, 208, 288, 352 rows: block boundaries
             (6, 58), (40, 9), (48, 9), (23, 22), (56, 9),                  # 354, 400, 480, 529, 560 rows: two equal tiles, 6 .. 9
             (60, 9), (62, 9), (64, 10),                                    # 600, 620, 704 rows: two full tiles
             (47, 14), (80, 9), (88, 9), (100, 9), (104, 10)]               # 705, 800, 880, 1000, 1144 rows: three and four tiles
    seen = set()
    for B, M in cases:
        R = B * (M + 1)
        form = plan(R)
        seen.add(form)
        shape = VerifyShape(f"tiles352_{dtype}_R{R}", B, M, 144, 600, dtype, 1.2)
        print(f"[case] {shape.name} {form}", flush=True)
        x = make_inputs(shape, 12)
        compare(jd.run_once(x), oracle_for(x))
    assert {f[1] for f in seen if f[0] == "one"} == set(range(6, 12)), seen
    assert {f[1] for f in seen if f[0] == "equal"} == set(range(6, 11)), seen
    assert {("full", 11, 6), ("full", 11, 8), ("full", 11, 11)} <= seen, seen


def test_bruteforce_interval_edges_on_gpu(jd):
    # the V = 8, M = 3 enumeration of tests/test_oracle_pins.py (every accept interval and every
    # CDF interval probed 1e-6 inside both ends) through the HIP library, ~30 k sequences in one call
    import itertools
    import math
    from paper_2501_19309_amd import binding as jb
    from tests.test_oracle_pins import _brute_setup, _mass_after
    V, M, P, Q, jbits, Pt, Qt = _brute_setup()
    eps = 1e-6
    toks, us, want_m, want_tok = [], [], [], []
    for c in itertools.product(range(V), repeat=M):
        a = [min(1.0, Pt[j][c[j]] / Qt[j][c[j]]) for j in range(M)]
        for m in range(M + 1):
            if m < M and (jbits[m] or a[m] >= 1.0 - 2 * eps):
                continue
            u, ok = [], True
            for j in range(M):
                if j < m:
                    if not jbits[j] and a[j] - eps <= 0.0:
                        ok = False
                        break
                    u.append(0.999 if jbits[j] else a[j] - eps)
                elif j == m:
                    u.append(a[j] + eps)
                else:
                    u.append(0.123)
            if not ok:
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
    B = len(toks)
    emb = np.broadcast_to(np.log(P).astype(np.float32), (B, M + 1, V)).copy()
    ej = np.zeros((B, M + 1, V), dtype=np.float32)
    ej[:, 1:, 0] = np.where(np.array(jbits) > 0, 1.0, -1.0)
    wj = np.zeros(V, dtype=np.float32); wj[0] = 1.0
    x = {"emb": emb, "W": np.eye(V, dtype=np.float32), "w_judge": wj, "emb_judge": ej,
         "draft_tokens": np.asarray(toks, dtype=np.int32),
         "draft_probs": np.broadcast_to(Q.astype(np.float32), (B, M, V)).copy(),
         "uniforms": np.asarray(us, dtype=np.float32)}
    got = jd.run_once(x, draft_kind=jb.JD_DRAFT_PROBS)
    ref = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_probs"], x["uniforms"],
                    emb_judge=ej, draft_kind=vo.DRAFT_PROBS)
    assert np.array_equal(ref["accept_len"], np.array(want_m)) and np.array_equal(ref["next_token"], np.array(want_tok))
    rep = compare(got, ref)
    exact = (got["accept_len"] == np.array(want_m)) & (got["next_token"] == np.array(want_tok))
    print("brute force on GPU:", B, "probes,", int((~exact).sum()), "inside the near-tie bands", rep, flush=True)
    assert exact.mean() > 0.999


def test_config_C1(jd):
    for seed in (0, 1, 2):
        x = make_inputs(CONFIGS["C1"], seed)
        rep = compare(jd.run_once(x, want_probs=True), oracle_for(x, return_probs=True))
        print("C1", seed, rep, flush=True)


def test_standard_mode_and_delta_one(jd):
    from paper_2501_19309_amd import binding as jb
    shape = VerifyShape("t", 4, 6, 256, 1500, "bf16", 1.0)
    x = make_inputs(shape, 3)
    std = jd.run_once(x, mode=jb.JD_MODE_STANDARD)
    compare(std, oracle_for(x, mode=vo.MODE_STANDARD), mode_judge=False)
    d1 = jd.run_once(x, delta=1.0)
    assert np.array_equal(d1["accept_len"], std["accept_len"])
    assert np.array_equal(d1["next_token"], std["next_token"])
    assert not d1["z_judge"].any()
    jud = jd.run_once(x)
    assert (jud["accept_len"] >= std["accept_len"]).all()
    # (0.999, 6.9) and (0.9999, 9.2): thresholds near logit(delta) where a float32 evaluation of the logit is off by
    # more than the judge band; the bias centres the judge logits on the threshold
    for delta, bias, T in [(0.8, 0.3, 1.0), (0.5, -0.2, 0.7), (0.6, 0.0, 1.6), (0.999, 6.9, 1.0), (0.9999, 9.2, 1.0)]:
        got = jd.run_once(x, delta=delta, judge_bias=bias, temperature=T)
        compare(got, oracle_for(x, delta=delta, judge_bias=bias, temperature=T))


def test_extreme_temperatures_and_logit_scales(jd):
    # Sharp and flat target distributions, and logits of magnitude ~1e3 (embeddings scaled up): the softmax
    # works around the row maximum, so nothing overflows and nothing underflows to a zero row sum.  Near-ties
    # are excluded by the comparison as everywhere; the point is that every other decision stays identical.
    for shape in (VerifyShape("x_skinny", 3, 7, 256, 2000, "bf16", 1.0), VerifyShape("x_gemm", 12, 10, 256, 2000, "bf16", 1.5),
                  VerifyShape("x_fp8", 2, 9, 256, 1200, "fp8", 1.0), VerifyShape("x_f32", 2, 4, 64, 300, "f32", 1.0)):
        x = make_inputs(shape, 4)
        for T in (0.02, 0.3, 25.0):
            rep = compare(jd.run_once(x, temperature=T, want_probs=True), oracle_for(x, temperature=T, return_probs=True))
            print(f"[case] {shape.name} T={T}", rep, flush=True)
        # embeddings 64 times larger (exact in bf16 and fp32: a power of two): logits in the hundreds
        xs = dict(x)
        if x["emb"].dtype == np.uint16:
            f = (x["emb"].astype(np.uint32) << np.uint32(16)).view(np.float32) * np.float32(64.0)
            xs["emb"] = bf16_bits_from_f32(f).reshape(x["emb"].shape)
        else:
            xs["emb"] = x["emb"] * np.float32(64.0)
        ref = oracle_for(xs, return_probs=True)
        got = jd.run_once(xs, want_probs=True)
        print(f"[case] {shape.name} x64", compare(got, ref), flush=True)
        assert np.isfinite(got["probs"]).all() and (got["status"] == 0).all()
        assert np.abs(got["probs"].astype(np.float64).sum(-1) - 1.0).max() < 1e-3


def test_probs_draft_and_dv_layout(jd):
    from paper_2501_19309_amd import binding as jb
    for kind in ("bf16", "f32"):
        shape = VerifyShape("t", 2, 5, 128, 777, kind, 1.0)
        x = make_inputs(shape, 5)
        D = x["draft_logits"].astype(np.float64)
        Q = np.exp(D - D.max(-1, keepdims=True)); Q /= Q.sum(-1, keepdims=True)
        x["draft_probs"] = Q.astype(np.float32)
        ref = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_probs"], x["uniforms"],
                        draft_kind=vo.DRAFT_PROBS)
        compare(jd.run_once(x, draft_kind=jb.JD_DRAFT_PROBS), ref)
        # [d][V] weight layout gives identical results to [V][d]
        xt = dict(x); xt["W"] = np.ascontiguousarray(x["W"].T)
        a = jd.run_once(x); b = jd.run_once(xt, w_layout=jb.JD_W_DV)
        for k in ("accept_len", "next_token", "z_stand", "z_judge", "p_at_draft", "judge_logit"):
            assert np.array_equal(a[k], b[k]), k


def test_topk_rule_and_target_resampling(jd):
    # Sec. 5 top-K verification (K = 1: greedy matching of Sec. 3.2) with greedy replacement, and the
    # literal "sample from p_i" replacement, against the oracle
    from paper_2501_19309_amd import binding as jb
    for kind, V in (("bf16", 3000), ("f32", 700)):
        shape = VerifyShape("t", 6, 8, 128, V, kind, 0.7)
        x = make_inputs(shape, 13)
        for K in (1, 4, 50, V):
            for mode, vmode in ((jb.JD_MODE_STANDARD, vo.MODE_STANDARD), (jb.JD_MODE_JUDGE, vo.MODE_JUDGE)):
                got = jd.run_once(x, rule=jb.JD_RULE_TOPK, top_k=K, mode=mode)
                ref = oracle_for(x, rule=vo.RULE_TOPK, top_k=K, mode=vmode)
                rep = compare(got, ref, mode_judge=(mode == jb.JD_MODE_JUDGE), rule_topk=True)
            if K == V:
                assert got["z_stand"].all()
        got = jd.run_once(x, resample=jb.JD_RESAMPLE_TARGET, mode=jb.JD_MODE_STANDARD)
        ref = oracle_for(x, resample=vo.RESAMPLE_TARGET, mode=vo.MODE_STANDARD)
        compare(got, ref, mode_judge=False)
        assert (ref["accept_len"] < 8).any()
    # exact ties: small-integer embeddings and weights give many equal logits; order is by token id
    rng = np.random.default_rng(3)
    for kind in ("bf16", "f32"):
        B, M, d, V = 5, 6, 32, 400
        emb = rng.integers(-2, 3, size=(B, M + 1, d)).astype(np.float32)
        W = rng.integers(-1, 2, size=(V, d)).astype(np.float32)
        Lint = np.einsum("brk,vk->brv", emb, W)                        # exact small integers
        top = Lint[:, :M].max(-1, keepdims=True)
        # draft the HIGHEST id among the tokens tied for the row maximum: whether it is accepted
        # at K = 1 depends only on the tie order (lower id ranks first)
        toks = (V - 1 - np.argmax((Lint[:, :M] == top)[..., ::-1], axis=-1)).astype(np.int32)
        assert ((Lint[:, :M] == top).sum(-1) > 1).any()
        x = {"emb": emb, "W": W, "w_judge": rng.integers(-1, 2, size=d).astype(np.float32),
             "draft_tokens": toks,
             "draft_logits": rng.normal(size=(B, M + 1, V)).astype(np.float32),
             "uniforms": rng.random((B, M + 1)).astype(np.float32)}
        if kind == "bf16":
            from synth import bf16_bits_from_f32
            for k in ("emb", "W", "w_judge"):
                x[k] = bf16_bits_from_f32(x[k]).reshape(x[k].shape)
        for K in (1, 3, 40):
            got = jd.run_once(x, rule=jb.JD_RULE_TOPK, top_k=K, mode=jb.JD_MODE_STANDARD)
            ref = oracle_for(x, rule=vo.RULE_TOPK, top_k=K, mode=vo.MODE_STANDARD)
            # logits are exact integers on both sides: no band is needed, everything must agree
            assert np.array_equal(got["z_stand"], ref["z_stand"]) and np.array_equal(got["accept_len"], ref["accept_len"])
            assert np.array_equal(got["next_token"], ref["next_token"])
            if K == 1:                                  # the case really contains ties at the boundary,
                assert (ref["accept_margin"] == 0).any() and not ref["z_stand"].all()   # decided by token id


def _random_shapes(n, seed):
    """Seeded shapes drawn over the dispatch boundaries: row counts on both sides of 64, 176, 352 and 704,
    hidden sizes with and without a ragged last K chunk, vocabularies with a ragged last group."""
    rng = np.random.default_rng(seed)
    shapes = []
    row_targets = [3, 17, 40, 63, 64, 65, 100, 175, 176, 177, 260, 351, 352, 353, 500, 529, 703, 704, 705, 900]
    for i in range(n):
        dtype = ("bf16", "fp8", "int8", "bf16", "f32")[i % 5]
        M = int(rng.integers(1, 21))
        B = max(1, int(row_targets[i % len(row_targets)] // (M + 1)))
        step = {"bf16": 8, "fp8": 16, "int8": 16, "f32": 1}[dtype]
        d = int(rng.integers(1, 48)) * step if dtype != "f32" else int(rng.integers(5, 90))
        V = int(rng.integers(65, 2600)) if dtype != "f32" else int(rng.integers(9, 700))
        if dtype == "f32":
            B = min(B, 12)
        noise = float(rng.uniform(0.5, 2.5))
        shapes.append(VerifyShape(f"r{i}_{dtype}_B{B}_M{M}_d{d}_V{V}", B, M, d, V, dtype, noise))
    return shapes


@pytest.mark.parametrize("shape", _random_shapes(40, 20250119), ids=lambda s: s.name)
def test_random_shapes_match_oracle(jd, shape):
    print(f"[case] {shape.name} R={shape.R}", flush=True)
    x = make_inputs(shape, 11)
    rep = compare(jd.run_once(x, want_probs=True), oracle_for(x, return_probs=True))
    print(rep, flush=True)


FP8 = [
    VerifyShape("q_1blk", 1, 5, 256, 1024, "fp8", 1.0),
    VerifyShape("q_2blk", 1, 25, 512, 2048, "fp8", 1.0),
    VerifyShape("q_ragged", 2, 9, 272, 1000, "fp8", 2.0),        # d % 256 != 0, V % 64 != 0
    VerifyShape("q_4blk", 4, 15, 768, 3000, "fp8", 1.5),         # R = 64
    VerifyShape("q_gemm", 9, 10, 512, 5000, "fp8", (0.5, 2.5)),  # R = 99: 176-row tiling, FP8 codes converted in registers
    VerifyShape("q_gemm176x3", 40, 10, 784, 3333, "fp8", (0.5, 2.5)),  # R = 440: two row tiles of 224 rows (352-row kernel), ragged d and V
    VerifyShape("q_gemm352", 20, 10, 288, 2100, "fp8", (0.5, 2.5)),  # R = 220: 352-row tiling, FP8 fragments
    VerifyShape("q_gemm704", 64, 10, 528, 4100, "fp8", (0.5, 2.5)),  # R = 704: two 352-row tiles, ragged d and V
    VerifyShape("q_gemm_d16", 33, 10, 16, 130, "fp8", 1.0),          # R = 363: two tiles, one real K step
    VerifyShape("q_d16", 2, 3, 16, 200, "fp8", 1.0),             # smallest hidden size of the FP8 path
]


@pytest.mark.parametrize("shape", FP8, ids=lambda s: s.name)
def test_fp8_weights_match_oracle(jd, shape):
    print(f"[case] {shape.name}", flush=True)
    for seed in (0, 1):
        x = make_inputs(shape, seed)
        rep = compare(jd.run_once(x, want_probs=True), oracle_for(x, return_probs=True))
        print(rep, flush=True)


def test_fp8_decode_of_every_code(jd):
    # logits[v] = scale * decode(code v): one code per vocabulary entry, a one-hot embedding.
    # Pins the hardware conversion (OCP E4M3: bias 7, subnormals, no infinities) against the table.
    V, d = 256, 32
    codes = np.arange(V, dtype=np.uint8); codes[0x7F] = 0x3A; codes[0xFF] = 0xBA   # skip the two NaN codes
    W = np.zeros((V, d), dtype=np.uint8); W[:, 5] = codes
    from synth import bf16_bits_from_f32
    for R_rows, M in ((2, 1), (70, 9)):                                             # small-row and GEMM regime
        B = R_rows // (M + 1)
        emb = np.zeros((B, M + 1, d), dtype=np.float32); emb[:, :, 5] = 1.0
        rng = np.random.default_rng(0)
        x = {"emb": bf16_bits_from_f32(emb).reshape(emb.shape), "W": W,
             "w_scale": np.full(V, 1.0 / 64, dtype=np.float32) * (1 + np.arange(V, dtype=np.float32) / 1024),
             "w_judge": bf16_bits_from_f32(np.ones(d, dtype=np.float32)),
             "draft_tokens": rng.integers(0, V, size=(B, M)).astype(np.int32),
             "draft_logits": rng.normal(size=(B, M + 1, V)).astype(np.float32),
             "uniforms": rng.random((B, M + 1)).astype(np.float32)}
        ref = oracle_for(x, return_probs=True)
        got = jd.run_once(x, want_probs=True)
        compare(got, ref)
        want = np.log(ref["probs"][0, 0]); have = np.log(got["probs"][0, 0].astype(np.float64))
        assert np.abs((have - have[0x38]) - (want - want[0x38])).max() < 1e-5   # logit differences, all 254 codes
    # a NaN code anywhere in a used weight row raises the NaN status
    Wn = W.copy(); Wn[17, 5] = 0x7F
    x["W"] = Wn
    got = jd.run_once(x)
    assert (got["status"].astype(np.int64) & 2).all()


INT8 = [
    VerifyShape("i_1blk", 1, 5, 256, 1024, "int8", 1.0),
    VerifyShape("i_2blk", 1, 25, 512, 2048, "int8", 1.0),
    VerifyShape("i_ragged", 2, 9, 272, 1000, "int8", 2.0),           # d % 256 != 0, V % 64 != 0
    VerifyShape("i_3blk", 4, 10, 768, 3000, "int8", 1.5),            # R = 44
    VerifyShape("i_4blk", 4, 15, 768, 3000, "int8", 1.5),            # R = 64
    VerifyShape("i_gemm", 9, 10, 512, 5000, "int8", (0.5, 2.5)),     # R = 99: one 176-row tile, codes converted in registers
    VerifyShape("i_gemm352", 20, 10, 288, 2100, "int8", (0.5, 2.5)), # R = 220: 352-row tiling on the bf16 copy
    VerifyShape("i_d16", 2, 3, 16, 200, "int8", 1.0),                # smallest hidden size of the 8-bit path
]


@pytest.mark.parametrize("shape", INT8, ids=lambda s: s.name)
def test_int8_weights_match_oracle(jd, shape):
    print(f"[case] {shape.name}", flush=True)
    for seed in (0, 1):
        x = make_inputs(shape, seed)
        rep = compare(jd.run_once(x, want_probs=True), oracle_for(x, return_probs=True))
        print(rep, flush=True)
    if shape.name in ("i_ragged", "i_gemm"):   # the [d, V] storage order of the same weights gives the same call
        from paper_2501_19309_amd import binding as jb
        xt = dict(x); xt["W"] = np.ascontiguousarray(x["W"].T)
        a = jd.run_once(x); b = jd.run_once(xt, w_layout=jb.JD_W_DV)
        for k in ("accept_len", "next_token", "z_stand", "z_judge", "p_at_draft", "judge_logit"):
            assert np.array_equal(a[k], b[k]), k


def test_int8_decode_of_every_code(jd):
    # logits[v] = scale[v] * code v: one bit pattern per vocabulary entry, a one-hot embedding, compared as
    # logit differences for all 256 patterns in the small-row kernel (codes converted in registers) and in
    # the large-row regime (bf16 copy)
    V, d = 256, 32
    W = np.zeros((V, d), dtype=np.int8); W[:, 5] = np.arange(V, dtype=np.uint8).view(np.int8)
    from synth import bf16_bits_from_f32
    for R_rows, M in ((2, 1), (70, 9)):
        B = R_rows // (M + 1)
        emb = np.zeros((B, M + 1, d), dtype=np.float32); emb[:, :, 5] = 1.0
        rng = np.random.default_rng(0)
        x = {"emb": bf16_bits_from_f32(emb).reshape(emb.shape), "W": W,
             "w_scale": np.full(V, 1.0 / 32, dtype=np.float32) * (1 + np.arange(V, dtype=np.float32) / 1024),
             "w_judge": bf16_bits_from_f32(np.ones(d, dtype=np.float32)),
             "draft_tokens": rng.integers(0, V, size=(B, M)).astype(np.int32),
             "draft_logits": rng.normal(size=(B, M + 1, V)).astype(np.float32),
             "uniforms": rng.random((B, M + 1)).astype(np.float32)}
        ref = oracle_for(x, return_probs=True)
        got = jd.run_once(x, want_probs=True)
        compare(got, ref)
        want = np.log(ref["probs"][0, 0]); have = np.log(got["probs"][0, 0].astype(np.float64))
        assert np.abs((have - have[1]) - (want - want[1])).max() < 1e-5


def test_separate_judge_embedding(jd):
    shape = VerifyShape("t", 3, 6, 256, 900, "bf16", 1.0)
    x = make_inputs(shape, 7)
    ej = make_inputs(shape, 8)["emb"]
    x["emb_judge"] = ej
    ref = oracle_for(x, emb_judge=ej)
    compare(jd.run_once(x), ref)
    base = jd.run_once({k: v for k, v in x.items() if k != "emb_judge"})
    assert not np.array_equal(base["judge_logit"], ref["judge_logit"].astype(np.float32))


def test_masked_draft_logits(jd):
    # a filtered draft distribution: logits of -inf (probability zero), also at the start of every column
    # range the statistics pass splits a row into, and on a drafted token itself (q[c] = 0: Eq. 4 then
    # accepts iff p[c] > 0)
    for shape in (VerifyShape("m_skinny", 3, 6, 256, 3001, "bf16", 1.0), VerifyShape("m_gemm", 9, 10, 256, 5000, "bf16", 1.5),
                  VerifyShape("m_f32", 2, 4, 64, 515, "f32", 1.0)):
        x = make_inputs(shape, 6)
        D = x["draft_logits"].copy()
        rng = np.random.default_rng(1)
        mask = rng.random(D.shape) < 0.3
        mask[..., :min(700, shape.V // 4)] = True   # a long run of masked tokens from column 0 on
        for b in range(shape.B):          # drafted tokens keep their mass ...
            for j in range(shape.M):
                mask[b, j, x["draft_tokens"][b, j]] = False
        mask[0, 1, x["draft_tokens"][0, 1]] = True   # ... except one
        D[mask] = -np.inf
        x["draft_logits"] = D
        ref = oracle_for(x)
        got = jd.run_once(x)
        rep = compare(got, ref)
        assert (ref["status"] == 0).all() and (got["status"] == 0).all(), (ref["status"], got["status"])
        assert got["q_at_draft"][0, 1] == 0.0 and got["z_stand"][0, 1] == 1
        print(shape.name, rep, flush=True)


def test_status_bits(jd):
    shape = VerifyShape("t", 4, 5, 128, 640, "bf16", 1.0)
    x = make_inputs(shape, 9)
    x["draft_tokens"] = x["draft_tokens"].copy()
    x["draft_tokens"][1, 2] = shape.V
    x["draft_tokens"][2, 0] = -5
    x["draft_logits"] = x["draft_logits"].copy()
    x["draft_logits"][3, 1, 17] = np.nan
    ref = oracle_for(x)
    got = jd.run_once(x)
    assert (got["status"].astype(np.int64) & 0xFFFFFFFF).tolist() == ref["status"].tolist() == [0, 1, 1, 2]
    for b in (0, 1, 2):
        assert int(got["accept_len"][b]) == int(ref["accept_len"][b])
        assert int(got["next_token"][b]) == int(ref["next_token"][b])
    # a draft row with every token masked (-inf) is no distribution (Eq. 3): reported like a NaN
    x["draft_logits"][3, 1, 17] = 0.5
    x["draft_logits"][0, 2, :] = -np.inf
    ref = oracle_for(x)
    got = jd.run_once(x)
    assert (got["status"].astype(np.int64) & 0xFFFFFFFF).tolist() == ref["status"].tolist() == [2, 1, 1, 0]
    # draft == target logits: q == p, no residual mass at a forced rejection -> flag + sample from p
    y = make_inputs(VerifyShape("t", 2, 4, 64, 512, "f32", 1.0), 1)
    L = vo.target_logits(y["emb"].reshape(-1, 64), y["W"]).reshape(2, 5, 512)
    y["draft_logits"] = L.astype(np.float32)
    y["draft_tokens"] = y["draft_tokens"].copy(); y["draft_tokens"][0, 1] = 10 ** 6
    ref = oracle_for(y, mode=vo.MODE_STANDARD)
    from paper_2501_19309_amd import binding as jb
    got = jd.run_once(y, mode=jb.JD_MODE_STANDARD)
    assert int(ref["status"][0]) & vo.STATUS_BAD_TOKEN
    assert int(got["accept_len"][0]) == 1 == int(ref["accept_len"][0])
    assert int(got["status"][0]) & 1
    # draft handed over as probabilities: a NaN in the row of the first rejection, away from the drafted token,
    # reaches only the sampler, which must report it instead of falling back to p silently
    z = make_inputs(VerifyShape("t", 3, 4, 64, 512, "bf16", 1.0), 5)
    D = z["draft_logits"].astype(np.float64)
    Q = np.exp(D - D.max(-1, keepdims=True)); Q /= Q.sum(-1, keepdims=True)
    z["draft_probs"] = Q.astype(np.float32)
    clean = vo.verify(z["emb"], z["W"], z["w_judge"], z["draft_tokens"], z["draft_probs"], z["uniforms"],
                      draft_kind=vo.DRAFT_PROBS)
    b = int(np.argmax(clean["accept_len"] < 4))
    m = int(clean["accept_len"][b])
    assert m < 4, "the workload must hold a rejection"
    c = int(z["draft_tokens"][b, m])
    z["draft_probs"][b, m, (c + 100) % 512] = np.nan
    ref = vo.verify(z["emb"], z["W"], z["w_judge"], z["draft_tokens"], z["draft_probs"], z["uniforms"],
                    draft_kind=vo.DRAFT_PROBS)
    got = jd.run_once(z, draft_kind=jb.JD_DRAFT_PROBS)
    assert int(ref["status"][b]) == vo.STATUS_NAN and int(got["status"][b]) == jb.JD_STATUS_NAN
    assert int(got["accept_len"][b]) == m
    others = [i for i in range(3) if i != b]
    assert (got["status"][others] == 0).all() and (ref["status"][others] == 0).all()


@pytest.mark.parametrize("shape", [VerifyShape("rel_bf16", 2, 9, 264, 3000, "bf16", 1.0),
                                   VerifyShape("rel_bf16_rows352", 32, 10, 256, 2100, "bf16", 1.0),
                                   VerifyShape("rel_bf16_rows200", 20, 9, 256, 2100, "bf16", 1.0),
                                   VerifyShape("rel_fp8", 3, 7, 256, 2000, "fp8", 1.5),
                                   VerifyShape("rel_fp8_rows352", 32, 10, 256, 2100, "fp8", 1.0),
                                   VerifyShape("rel_int8", 3, 7, 256, 2000, "int8", 1.5),
                                   VerifyShape("rel_int8_rows352", 32, 10, 256, 2100, "int8", 1.0)], ids=lambda s: s.name)
def test_caller_weights_may_be_released_after_create(jd, shape):
    # bf16 and 8-bit contexts work from the library's own re-tiled copies: once create has returned, the caller's
    # W_lm is not read again.  Here it is overwritten with NaN patterns before the call.
    import torch
    from paper_2501_19309_amd import harness
    x = make_inputs(shape, 6)
    dev = harness.to_device(x)
    ver = harness.make_verifier(dev)
    try:
        W = dev["W"]
        if W.dtype == torch.bfloat16:
            W.view(torch.int16).fill_(0x7FC0)      # bf16 quiet NaN
        elif W.dtype == torch.uint8:
            W.fill_(0x7F)                          # E4M3 NaN
        else:
            W.fill_(-128)                          # INT8: a valid code, but not the model's
        torch.cuda.synchronize()
        out = ver.alloc_outputs(shape.B, shape.M)
        ver.run(dev["emb"], dev["draft_tokens"], dev["draft_logits"], dev["uniforms"], out)
        torch.cuda.synchronize()
        print(shape.name, compare(out.to_numpy(), oracle_for(x)), flush=True)
    finally:
        ver.destroy()


def test_determinism_and_context_reuse(jd):
    import torch
    from paper_2501_19309_amd import harness
    big = make_inputs(VerifyShape("t", 4, 10, 512, 3000, "bf16", 1.0), 11)
    small = make_inputs(VerifyShape("t", 2, 4, 512, 3000, "bf16", 1.0), 12)
    small["W"], small["w_judge"] = big["W"], big["w_judge"]
    dev_big, dev_small = harness.to_device(big), harness.to_device(small)
    ver = harness.make_verifier(dev_big)
    try:
        outs = []
        for rep in range(3):
            o = ver.alloc_outputs(4, 10)
            ver.run(dev_big["emb"], dev_big["draft_tokens"], dev_big["draft_logits"], dev_big["uniforms"], o)
            torch.cuda.synchronize()
            outs.append(o.to_numpy())
            # a smaller call on the same context in between (B < max_B, M < max_M)
            o2 = ver.alloc_outputs(2, 4)
            ver.run(dev_small["emb"], dev_small["draft_tokens"], dev_small["draft_logits"], dev_small["uniforms"], o2)
            torch.cuda.synchronize()
            compare(o2.to_numpy(), oracle_for(small))
        for o in outs[1:]:
            for k, v in outs[0].items():
                assert np.array_equal(v, o[k], equal_nan=True), k
        compare(outs[0], oracle_for(big))
    finally:
        ver.destroy()


def test_side_stream_and_two_contexts(jd):
    # work is enqueued on the stream the caller passes (here a non-default one, default priority), and two
    # contexts with different shapes live side by side without disturbing each other
    import torch
    from paper_2501_19309_amd import harness
    xa = make_inputs(VerifyShape("a", 3, 9, 264, 3000, "bf16", 1.0), 31)     # small-row regime
    xb = make_inputs(VerifyShape("b", 20, 10, 256, 2100, "bf16", 1.5), 32)   # 352-row tiles
    da, db = harness.to_device(xa), harness.to_device(xb)
    va, vb = harness.make_verifier(da), harness.make_verifier(db)
    try:
        oa, ob = va.alloc_outputs(3, 9), vb.alloc_outputs(20, 10)
        side = torch.cuda.Stream()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            for _ in range(3):   # interleaved, all on the side stream
                va.run(da["emb"], da["draft_tokens"], da["draft_logits"], da["uniforms"], oa)
                vb.run(db["emb"], db["draft_tokens"], db["draft_logits"], db["uniforms"], ob)
        side.synchronize()
        compare(oa.to_numpy(), oracle_for(xa))
        compare(ob.to_numpy(), oracle_for(xb))
        # the same calls on the default stream give the same bits
        ga, gb = oa.to_numpy(), ob.to_numpy()
        va.run(da["emb"], da["draft_tokens"], da["draft_logits"], da["uniforms"], oa)
        vb.run(db["emb"], db["draft_tokens"], db["draft_logits"], db["uniforms"], ob)
        torch.cuda.synchronize()
        for k, v in oa.to_numpy().items():
            assert np.array_equal(v, ga[k], equal_nan=True), k
        for k, v in ob.to_numpy().items():
            assert np.array_equal(v, gb[k], equal_nan=True), k
    finally:
        va.destroy(); vb.destroy()


@pytest.mark.parametrize("shape", [VerifyShape("g_skinny", 2, 9, 264, 3000, "bf16", 1.0),
                                   VerifyShape("g_gemm", 20, 10, 256, 2100, "bf16", 1.5),
                                   VerifyShape("g_176", 9, 10, 256, 2100, "bf16", 1.5),
                                   VerifyShape("g_fp8_352", 32, 10, 272, 2100, "fp8", 1.5),
                                   VerifyShape("g_two_launches", 60, 9, 256, 2100, "bf16", 1.5)],   # 600 rows: a full row tile + a ragged one of its own
                         ids=lambda s: s.name)
def test_graph_capture_and_replay(jd, shape):
    # a serving loop may capture verify + append into a HIP graph: run() allocates nothing, never synchronises and
    # sets no function attributes, so it can be captured; every replay (with eager work and synchronisations between
    # them, and fresh inputs copied into the captured buffers) must equal the eager result and the oracle
    import torch
    from paper_2501_19309_amd import binding as jb, harness
    xs = [make_inputs(shape, 40 + k, prenorm=True, weights_seed=40) for k in range(2)]
    dev = harness.to_device(xs[0])
    ver = harness.make_verifier(dev)
    try:
        B, M = shape.B, shape.M
        out = ver.alloc_outputs(B, M)
        cap = 4 * (M + 1)
        buf = torch.zeros(B, cap, dtype=torch.int32, device="cuda"); lengths = torch.zeros(B, dtype=torch.int32, device="cuda")
        eps = float(xs[0]["rms_eps"])

        def call():
            ver.run_prenorm(dev["hidden"], dev["gamma"], eps, dev["draft_tokens"], dev["draft_logits"], dev["uniforms"], out)
            jb.append_tokens(dev["draft_tokens"], out.accept_len, out.next_token, buf, lengths)

        call()                       # eager once (also warms everything up)
        torch.cuda.synchronize()
        eager0 = out.to_numpy()
        buf.zero_(); lengths.zero_()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            call()
        rbuf = np.zeros((B, cap), dtype=np.int32); rlen = np.zeros(B, dtype=np.int64)
        buf.zero_(); lengths.zero_()
        for it, k in enumerate((0, 1, 0)):
            x = xs[k]
            fresh = harness.to_device({n: x[n] for n in ("hidden", "draft_tokens", "draft_logits", "uniforms")})
            for n, t in fresh.items():
                dev[n].copy_(t)      # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            got = out.to_numpy()
            ref = prenorm_oracle(x)
            compare(got, ref)
            if k == 0:
                for name, v in got.items():
                    assert np.array_equal(v, eager0[name], equal_nan=True), (it, name)
            vo.append_tokens(rbuf, rlen, x["draft_tokens"], got["accept_len"], got["next_token"])
            assert np.array_equal(lengths.cpu().numpy(), rlen) and np.array_equal(buf.cpu().numpy(), rbuf), it
    finally:
        ver.destroy()


@pytest.mark.parametrize("shape", [VerifyShape("p_skinny", 5, 9, 264, 3000, "bf16", 1.0),
                                   VerifyShape("p_gemm", 36, 10, 256, 2100, "bf16", 1.5)], ids=lambda s: s.name)
def test_batch_order_and_truncated_drafts_on_gpu(jd, shape):
    # sequences are independent: permuting the batch permutes every output bit for bit (a row's arithmetic
    # does not depend on where it sits in a tile); verifying only the first M' drafted tokens reproduces the
    # masks on those slots and cuts the prefix at M'
    x = make_inputs(shape, 17)
    got = jd.run_once(x)
    perm = np.random.default_rng(5).permutation(shape.B)
    y = dict(x)
    for k in ("emb", "draft_tokens", "draft_logits", "uniforms"):
        y[k] = np.ascontiguousarray(x[k][perm])
    gotp = jd.run_once(y)
    for k, v in got.items():
        assert np.array_equal(gotp[k], v[perm], equal_nan=True), k
    Mp = 4
    z = dict(x)
    z["emb"] = np.ascontiguousarray(x["emb"][:, :Mp + 1]); z["draft_tokens"] = np.ascontiguousarray(x["draft_tokens"][:, :Mp])
    z["draft_logits"] = np.ascontiguousarray(x["draft_logits"][:, :Mp + 1])
    z["uniforms"] = np.ascontiguousarray(np.concatenate([x["uniforms"][:, :Mp], x["uniforms"][:, shape.M:]], axis=1))
    gott = jd.run_once(z)
    compare(gott, oracle_for(z))
    ref = oracle_for(x)
    firm = (ref["accept_margin"][:, :Mp] > 1e-4).all(axis=1)     # away from ties the two launches must agree exactly
    assert firm.sum() >= shape.B - 1
    assert np.array_equal(gott["z_stand"][firm], got["z_stand"][firm][:, :Mp])
    assert np.array_equal(gott["accept_len"][firm], np.minimum(got["accept_len"], Mp)[firm])


def test_outputs_stay_inside_their_buffers(jd):
    # Every output tensor sits between two guard zones filled with a sentinel; the context is sized for a
    # larger batch than the call.  The call must write exactly its B x M (+1) elements and nothing beyond.
    import torch
    from paper_2501_19309_amd import binding as jb, harness
    G = 96
    for shape, big in ((VerifyShape("g_skinny", 3, 7, 256, 1111, "bf16", 1.0), (5, 9)),
                       (VerifyShape("g_gemm", 30, 10, 264, 1111, "bf16", 1.5), (40, 12)),
                       (VerifyShape("g_fp8", 20, 9, 272, 900, "fp8", 1.0), (33, 10)),
                       (VerifyShape("g_f32", 2, 4, 64, 300, "f32", 1.0), (3, 6))):
        x = make_inputs(shape, 9)
        B, M, V = shape.B, shape.M, shape.V
        dev = harness.to_device(x)
        ver = harness.make_verifier(dev, max_B=big[0], max_M=big[1])
        try:
            plain = ver.alloc_outputs(B, M, True)
            ver.run(dev["emb"], dev["draft_tokens"], dev["draft_logits"], dev["uniforms"], plain)
            guarded, backing = {}, {}
            for name, t in plain.__dict__.items():
                sentinel = 0x5A if t.dtype == torch.uint8 else (-123456789 if t.dtype == torch.int32 else -7.25)
                buf = torch.full((t.numel() + 2 * G,), sentinel, dtype=t.dtype, device=t.device)
                backing[name] = (buf, sentinel)
                guarded[name] = buf[G:G + t.numel()].view(t.shape)
                assert guarded[name].is_contiguous()
            out = jb.VerifyOutputs(**guarded)
            ver.run(dev["emb"], dev["draft_tokens"], dev["draft_logits"], dev["uniforms"], out)
            torch.cuda.synchronize()
            for name, (buf, sentinel) in backing.items():
                assert bool((buf[:G] == sentinel).all()) and bool((buf[-G:] == sentinel).all()), (shape.name, name)
                assert torch.equal(guarded[name], getattr(plain, name)), (shape.name, name)
        finally:
            ver.destroy()


CABI = [
    (VerifyShape("c_skinny", 2, 7, 512, 4000, "bf16", 1.0), False),
    (VerifyShape("c_gemm176", 9, 10, 264, 5000, "bf16", (0.5, 2.5)), True),
    (VerifyShape("c_gemm352", 32, 10, 512, 2100, "bf16", (0.5, 2.0)), False),
    (VerifyShape("c_fp8", 3, 9, 272, 3000, "fp8", 1.0), True),
    (VerifyShape("c_int8", 20, 10, 256, 1500, "int8", 1.5), False),
    (VerifyShape("c_f32", 2, 4, 64, 515, "f32", 1.0), False),
]


@pytest.mark.parametrize("shape,prenorm", CABI, ids=lambda v: v.name if isinstance(v, VerifyShape) else str(v))
def test_c_abi_from_plain_cpp_matches_oracle(shape, prenorm, tmp_path):
    # The library called from a C++ program of its own process (tests/cabi_check.cpp, built by build()): no Python
    # and no torch in that process.  Tensors travel as raw files; the outputs meet the same parity bar.
    import subprocess
    from paper_2501_19309_amd import binding as jb
    from paper_2501_19309_amd.build import CABI_CHECK_PATH
    import os
    assert os.path.exists(CABI_CHECK_PATH), "jd_cabi_check is not built: run __graft_entry__.build()"
    x = make_inputs(shape, 5, prenorm=prenorm)
    for name in ("emb", "hidden", "gamma", "W", "w_judge", "w_scale", "draft_logits", "draft_tokens", "uniforms"):
        if name in x:
            np.ascontiguousarray(x[name]).tofile(tmp_path / f"{name}.bin")
    wdt = {"f32": jb.JD_F32, "bf16": jb.JD_BF16, "fp8": jb.JD_FP8_E4M3, "int8": jb.JD_INT8}[shape.dtype]
    cmd = [CABI_CHECK_PATH, str(tmp_path), str(shape.B), str(shape.M), str(shape.d), str(shape.V), str(wdt), str(int(prenorm))]
    print("[case]", " ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=100)
    print(res.stdout, res.stderr, flush=True)
    assert res.returncode == 0, res.stdout + res.stderr
    B, M = shape.B, shape.M
    kinds = {"accept_len": (np.int32, (B,)), "next_token": (np.int32, (B,)), "status": (np.uint32, (B,)),
             "z_stand": (np.uint8, (B, M)), "z_judge": (np.uint8, (B, M)), "p_at_draft": (np.float32, (B, M)),
             "q_at_draft": (np.float32, (B, M)), "judge_logit": (np.float32, (B, M)),
             "row_max": (np.float32, (B, M + 1)), "row_sumexp": (np.float32, (B, M + 1))}
    got = {k: np.fromfile(tmp_path / f"{k}.bin", dtype=dt).reshape(sh) for k, (dt, sh) in kinds.items()}
    kw = {"w_scale": x["w_scale"]} if "w_scale" in x else {}
    if prenorm:
        emb, _ = vo.rmsnorm_rows(x["hidden"], x["gamma"], x["rms_eps"])
        kw["emb_judge"] = x["hidden"]
    else:
        emb = x["emb"]
    ref = vo.verify(emb, x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"], **kw)
    print(compare(got, ref), flush=True)


def test_device_probes(jd):
    # diagnostics behind the C ABI: plausible numbers, argument errors
    import ctypes
    from paper_2501_19309_amd import binding as jb
    lib = jb.load_library()
    tf = jb.probe_mfma_bf16(0, 1)
    gbs = jb.probe_hbm_read(0, 2 << 30)
    gbs_plain = jb.probe_hbm_read(0, 2 << 30, plain_loads=True)
    tf32 = jb.probe_mfma_bf16(0, 2)
    print(f"[probe] mfma bf16 16x16x32 {tf:.0f} TFLOP/s, 32x32x16 {tf32:.0f} TFLOP/s, hbm read {gbs:.0f} GB/s "
          f"(plain loads {gbs_plain:.0f})", flush=True)
    assert 300.0 < tf <= 2600.0 and 1000.0 < gbs <= 8200.0      # below the published peaks, far above a broken loop
    assert 1000.0 < gbs_plain <= 8200.0
    assert 300.0 < tf32 <= 2600.0
    v = ctypes.c_double()
    assert lib.jd_verify_probe_mfma_bf16(0, 7, ctypes.byref(v)) == jb.JD_ERR_INVALID_ARG
    assert lib.jd_verify_probe_mfma_bf16(0, 1, None) == jb.JD_ERR_INVALID_ARG
    assert lib.jd_verify_probe_hbm_read(0, 1000, ctypes.byref(v)) == jb.JD_ERR_INVALID_ARG
    assert lib.jd_verify_probe_hbm_read(-1, 1 << 30, ctypes.byref(v)) == jb.JD_ERR_INVALID_ARG
    assert lib.jd_verify_probe_hbm_read_plain(0, 1000, ctypes.byref(v)) == jb.JD_ERR_INVALID_ARG


def test_bench_json_contract(repo_root):
    # bench.py prints ONE JSON line with the keys the harness reads; the smallest workload keeps this quick
    import json, subprocess, sys, os
    res = subprocess.run([sys.executable, os.path.join(repo_root, "bench.py"), "--config", "C1", "--steps", "5", "--warmup", "2"],
                         capture_output=True, text=True, timeout=110, cwd=repo_root)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines
    r = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in r, k
    assert r["n_gpus"] == 1 and r["steps"] == 5 and r["warmup"] == 2 and r["higher_is_better"] is True
    assert r["vs_baseline"] is None and r["data"] == "synthetic" and "workload" in r["config"]
    assert r["value"] > 0 and abs(r["value"] - 5 / (r["ms_per_step"] * 1e-3)) < 1e-6 * r["value"]   # B*M = 5 positions per call
    rf = r["roofline"]
    for k in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert k in rf, k
    assert rf["bound"] in ("hbm", "mfma", "alu") and abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9
    cb = r["cpu_baseline"]
    for k in ("value", "unit", "cores", "kind", "sample"):
        assert k in cb, k
    assert cb["kind"] == "oracle" and cb["value"] > 0 and r["parity"]["ok"] is True
    # more than one GPU is refused with a message
    res2 = subprocess.run([sys.executable, os.path.join(repo_root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                          timeout=60, cwd=repo_root)
    assert res2.returncode != 0 and "one GPU" in (res2.stdout + res2.stderr)


def test_create_destroy_returns_all_device_memory(jd):
    # every buffer a context allocates (re-tiled weights, logits, pooled row arrays, profiling events) goes back
    import torch
    from paper_2501_19309_amd import harness
    shapes = (VerifyShape("l_bf16", 40, 10, 512, 6000, "bf16", 1.0), VerifyShape("l_fp8", 40, 10, 512, 6000, "fp8", 1.0),
              VerifyShape("l_int8", 40, 10, 512, 6000, "int8", 1.0), VerifyShape("l_f32", 2, 4, 64, 515, "f32", 1.0))
    devs = [harness.to_device(make_inputs(sh, 1)) for sh in shapes]
    def one_round(it):
        for sh, dev in zip(shapes, devs):
            ver = harness.make_verifier(dev, rule=(1 if it % 2 else 0), top_k=3)
            out = ver.alloc_outputs(sh.B, sh.M)
            ver.profile_begin(2)
            ver.run(dev["emb"], dev["draft_tokens"], dev["draft_logits"], dev["uniforms"], out)
            torch.cuda.synchronize()
            ver.profile_end()
            ver.destroy()
            del out

    for it in range(2):      # first use loads the kernels' code and lets the runtime and torch set up their pools
        one_round(it)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    free0, _ = torch.cuda.mem_get_info()
    for it in range(12):
        one_round(it)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    free1, _ = torch.cuda.mem_get_info()
    assert free0 - free1 < (4 << 20), (free0, free1)   # nothing of the contexts' ~100 MB per round is left behind


def test_draft_tensor_without_the_bonus_row(jd):
    # the draft model has no distribution for the bonus position: a draft tensor of M rows per sequence
    # (draft_rows = M) gives the same call as one with an ignored trailing row, logits and probabilities alike
    from paper_2501_19309_amd import binding as jb
    for shape in (VerifyShape("dr_skinny", 3, 6, 256, 1500, "bf16", 1.0), VerifyShape("dr_gemm", 12, 10, 256, 1500, "bf16", 1.5),
                  VerifyShape("dr_fp8", 2, 9, 256, 1200, "fp8", 1.0), VerifyShape("dr_f32", 2, 4, 64, 300, "f32", 1.0)):
        x = make_inputs(shape, 8)
        M = shape.M
        xm = dict(x); xm["draft_logits"] = np.ascontiguousarray(x["draft_logits"][:, :M])
        assert xm["draft_logits"].shape[1] == M
        full = jd.run_once(x, want_probs=True)
        cut = jd.run_once(xm, want_probs=True)
        for k in full:
            assert np.array_equal(full[k], cut[k]), (shape.name, k)
        compare(cut, oracle_for(xm, return_probs=True))
        D = x["draft_logits"].astype(np.float64)
        Q = np.exp(D - D.max(-1, keepdims=True)); Q /= Q.sum(-1, keepdims=True)
        xq = dict(x); xq["draft_probs"] = np.ascontiguousarray(Q[:, :M].astype(np.float32))
        kw = {"w_scale": x["w_scale"]} if "w_scale" in x else {}
        ref = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], xq["draft_probs"], x["uniforms"],
                        draft_kind=vo.DRAFT_PROBS, **kw)
        compare(jd.run_once(xq, draft_kind=jb.JD_DRAFT_PROBS), ref)


def test_dv_weight_layout_for_every_weight_type(jd):
    # W_lm handed over as [d][V] (the transpose of the checkpoint layout): every re-tiling kernel and the fp32
    # LM head read it through their layout switch; same integer outputs and probabilities as [V][d]
    from paper_2501_19309_amd import binding as jb
    for shape in (VerifyShape("dv_fp8_skinny", 2, 9, 272, 1000, "fp8", 2.0),           # Wp8
                  VerifyShape("dv_fp8_176", 9, 10, 272, 1000, "fp8", (0.5, 2.5)),      # Wp8 in the 176-row kernel
                  VerifyShape("dv_fp8_352", 32, 10, 272, 1000, "fp8", (0.5, 2.5)),     # Wg8
                  VerifyShape("dv_int8_352", 32, 10, 272, 1000, "int8", (0.5, 2.5)),   # bf16 copy from INT8
                  VerifyShape("dv_bf16_352", 32, 10, 264, 1000, "bf16", (0.5, 2.5)),
                  VerifyShape("dv_f32", 3, 5, 100, 515, "f32", 1.0)):
        x = make_inputs(shape, 3)
        xt = dict(x); xt["W"] = np.ascontiguousarray(x["W"].T)
        a = jd.run_once(x, want_probs=True)
        b = jd.run_once(xt, want_probs=True, w_layout=jb.JD_W_DV)
        for k in a:
            assert np.array_equal(a[k], b[k]), (shape.name, k)
        ref = vo.verify(x["emb"], xt["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"],
                        w_layout="dv", return_probs=True, **({"w_scale": x["w_scale"]} if "w_scale" in x else {}))
        compare(b, ref)


def test_options_in_the_large_row_regime(jd):
    # the rule / mode / draft-kind / resampling switches on top of the 176-row and 352-row LM-head kernels
    from paper_2501_19309_amd import binding as jb
    for shape in (VerifyShape("o_176", 9, 10, 264, 2100, "bf16", (0.5, 2.5)), VerifyShape("o_352", 32, 10, 264, 2100, "bf16", (0.5, 2.5)),
                  VerifyShape("o_352_fp8", 32, 10, 272, 2100, "fp8", (0.5, 2.5))):
        x = make_inputs(shape, 21)
        kw = {"w_scale": x["w_scale"]} if "w_scale" in x else {}
        for K in (1, 5):
            got = jd.run_once(x, rule=jb.JD_RULE_TOPK, top_k=K)
            compare(got, oracle_for(x, rule=vo.RULE_TOPK, top_k=K), rule_topk=True)
        got = jd.run_once(x, resample=jb.JD_RESAMPLE_TARGET, mode=jb.JD_MODE_STANDARD, temperature=0.8)
        compare(got, oracle_for(x, resample=vo.RESAMPLE_TARGET, mode=vo.MODE_STANDARD, temperature=0.8), mode_judge=False)
        got = jd.run_once(x, delta=0.7, judge_bias=0.4)
        compare(got, oracle_for(x, delta=0.7, judge_bias=0.4))
        D = x["draft_logits"].astype(np.float64)
        Q = np.exp(D - D.max(-1, keepdims=True)); Q /= Q.sum(-1, keepdims=True)
        xq = dict(x); xq["draft_probs"] = Q.astype(np.float32)
        ref = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], xq["draft_probs"], x["uniforms"],
                        draft_kind=vo.DRAFT_PROBS, **kw)
        compare(jd.run_once(xq, draft_kind=jb.JD_DRAFT_PROBS), ref)
        ej = make_inputs(shape, 22)["emb"]
        xj = dict(x); xj["emb_judge"] = ej
        compare(jd.run_once(xj), oracle_for(x, emb_judge=ej))


def test_nan_status_in_every_lm_head_kernel(jd):
    # a NaN in one sequence's embeddings (bf16 0x7FC0) or in one weight row must raise that sequence's
    # (resp. every sequence's) NaN bit through the small-row, the 176-row and the 352-row LM-head kernels,
    # and leave the clean sequences' results as the oracle has them
    for shape in (VerifyShape("nan_skinny", 4, 9, 256, 1500, "bf16", 1.0), VerifyShape("nan_176", 9, 10, 256, 1500, "bf16", 1.0),
                  VerifyShape("nan_352", 32, 10, 256, 1500, "bf16", 1.0), VerifyShape("nan_352_fp8", 32, 10, 256, 1500, "fp8", 1.0)):
        x = make_inputs(shape, 17)
        x["emb"] = x["emb"].copy()
        x["emb"][2, 3, 100] = 0x7FC0            # row 3 of sequence 2: its LM-head row and judge slot 2 become NaN
        ref = oracle_for(x)
        got = jd.run_once(x)
        st = got["status"].astype(np.int64) & 0xFFFFFFFF
        assert st.tolist() == ref["status"].tolist(), shape.name
        assert st[2] & 2 and not (np.delete(st, 2) & 2).any()
        clean = [b for b in range(shape.B) if b != 2]
        assert np.array_equal(got["accept_len"][clean], ref["accept_len"][clean])
        assert np.array_equal(got["next_token"][clean], ref["next_token"][clean])
        if shape.dtype == "bf16":              # a NaN weight: every row's softmax is NaN
            y = make_inputs(shape, 17)
            y["W"] = y["W"].copy(); y["W"][777, 5] = 0x7FC0
            refy = oracle_for(y)
            goty = jd.run_once(y)
            assert (refy["status"] & 2).all() and ((goty["status"].astype(np.int64) & 2) != 0).all()


def test_run_argument_errors(jd):
    import ctypes
    from paper_2501_19309_amd import binding as jb, harness
    x = make_inputs(VerifyShape("t", 2, 4, 64, 256, "bf16", 1.0), 0)
    dev = harness.to_device(x)
    ver = harness.make_verifier(dev)
    try:
        o = ver.alloc_outputs(2, 4)
        outs = jb.jd_verify_outputs(o.accept_len.data_ptr(), o.next_token.data_ptr(), o.status.data_ptr())
        args = dict(emb=dev["emb"].data_ptr(), emb_judge=None, draft_tokens=dev["draft_tokens"].data_ptr(),
                    draft=dev["draft_logits"].data_ptr(), uniforms=dev["uniforms"].data_ptr())
        assert ver.run_raw(3, 4, draft_rows=5, outputs=outs, **args) == jb.JD_ERR_SHAPE
        assert ver.run_raw(2, 5, draft_rows=5, outputs=outs, **args) == jb.JD_ERR_SHAPE
        assert ver.run_raw(2, 4, draft_rows=3, outputs=outs, **args) == jb.JD_ERR_SHAPE
        assert ver.run_raw(0, 4, draft_rows=5, outputs=outs, **args) == jb.JD_ERR_SHAPE
        assert ver.run_raw(2, 4, draft_rows=5, outputs=None, **args) == jb.JD_ERR_INVALID_ARG
        bad = jb.jd_verify_outputs(o.accept_len.data_ptr(), None, o.status.data_ptr())
        assert ver.run_raw(2, 4, draft_rows=5, outputs=bad, **args) == jb.JD_ERR_INVALID_ARG
        args["emb"] = None
        assert ver.run_raw(2, 4, draft_rows=5, outputs=outs, **args) == jb.JD_ERR_INVALID_ARG
        assert ver.workspace_bytes() > 0
    finally:
        ver.destroy()
    assert jb.load_library().jd_verify_destroy(None) == jb.JD_OK


# ----------------------------------------------------------------------------- pre-norm wiring (Sec. 4.1)

PRENORM = [
    VerifyShape("n_f32", 3, 5, 100, 1000, "f32", 1.0),
    VerifyShape("n_bf16_skinny", 2, 9, 264, 1000, "bf16", 1.5),      # R = 20: judge rides beside the LM head
    VerifyShape("n_bf16_R64", 4, 15, 768, 3000, "bf16", 1.0),
    VerifyShape("n_bf16_gemm176", 9, 10, 512, 5000, "bf16", (0.5, 2.5)),   # R = 99
    VerifyShape("n_bf16_gemm352", 32, 10, 520, 4100, "bf16", (0.5, 2.0)),  # R = 352
    VerifyShape("n_fp8", 1, 25, 512, 2048, "fp8", 1.0),
]


def prenorm_oracle(x, **kw):
    emb, _ = vo.rmsnorm_rows(x["hidden"], x["gamma"], x["rms_eps"])
    return oracle_call(emb, x, emb_judge=x["hidden"], **kw)


@pytest.mark.parametrize("shape", PRENORM, ids=lambda s: s.name)
def test_prenorm_wiring_matches_oracle(jd, shape):
    print(f"[case] {shape.name}", flush=True)
    for seed in (0, 1):
        x = make_inputs(shape, seed, prenorm=True)
        ref = prenorm_oracle(x, return_probs=True)
        got = jd.run_once(x, want_probs=True)
        rep = compare(got, ref)
        print(rep, flush=True)


def test_prenorm_rounding_is_the_oracles(jd):
    # identity LM head: the logits ARE the normalised, rounded embeddings, so the probabilities give them
    # back to ~1e-6 while one bf16 step is 4e-3 relative: every rounding decision of the kernel is checked
    d = V = 1024
    shape = VerifyShape("t", 4, 15, d, V, "bf16", 1.0)
    x = make_inputs(shape, 2, prenorm=True)
    x["W"] = bf16_bits_from_f32(np.eye(V, dtype=np.float32))
    got = jd.run_once(x, want_probs=True)
    emb, _ = vo.rmsnorm_rows(x["hidden"], x["gamma"], x["rms_eps"])
    want = vo.widen(emb)
    back = np.log(got["probs"].astype(np.float64)) + np.log(got["row_sumexp"].astype(np.float64))[..., None] \
        + got["row_max"].astype(np.float64)[..., None]
    err = np.abs(back - want)
    print("max |recovered - oracle| =", err.max(), "; smallest bf16 step among the values:",
          (np.abs(want)[want != 0] * 2.0 ** -8).min(), flush=True)
    assert err.max() < 2e-5
    # the same through the fp32 path: rounded once to float32
    shape = VerifyShape("t", 2, 3, 64, 64, "f32", 1.0)
    x = make_inputs(shape, 3, prenorm=True)
    x["W"] = np.eye(64, dtype=np.float32)
    got = jd.run_once(x, want_probs=True)
    emb, _ = vo.rmsnorm_rows(x["hidden"], x["gamma"], x["rms_eps"])
    back = np.log(got["probs"].astype(np.float64)) + np.log(got["row_sumexp"].astype(np.float64))[..., None] \
        + got["row_max"].astype(np.float64)[..., None]
    assert np.abs(back - emb.astype(np.float64)).max() < 2e-5


def test_prenorm_argument_errors(jd):
    from paper_2501_19309_amd import binding as jb, harness
    x = make_inputs(VerifyShape("t", 2, 4, 64, 256, "bf16", 1.0), 0, prenorm=True)
    dev = harness.to_device(x)
    ver = harness.make_verifier(dev)
    try:
        o = ver.alloc_outputs(2, 4)
        outs = jb.jd_verify_outputs(o.accept_len.data_ptr(), o.next_token.data_ptr(), o.status.data_ptr())
        a = dict(hidden=dev["hidden"].data_ptr(), gamma=dev["gamma"].data_ptr(), rms_eps=1e-5,
                 draft_tokens=dev["draft_tokens"].data_ptr(), draft=dev["draft_logits"].data_ptr(), draft_rows=5,
                 uniforms=dev["uniforms"].data_ptr(), outputs=outs)
        assert ver.run_prenorm_raw(2, 4, **a) == jb.JD_OK
        assert ver.run_prenorm_raw(2, 4, **{**a, "gamma": None}) == jb.JD_ERR_INVALID_ARG
        assert ver.run_prenorm_raw(2, 4, **{**a, "hidden": None}) == jb.JD_ERR_INVALID_ARG
        assert ver.run_prenorm_raw(2, 4, **{**a, "rms_eps": -1e-5}) == jb.JD_ERR_INVALID_ARG
        assert ver.run_prenorm_raw(2, 4, **{**a, "rms_eps": float("nan")}) == jb.JD_ERR_INVALID_ARG
        assert ver.run_prenorm_raw(2, 4, **{**a, "rms_eps": float("inf")}) == jb.JD_ERR_INVALID_ARG
        assert ver.run_prenorm_raw(3, 4, **a) == jb.JD_ERR_SHAPE
        import torch
        torch.cuda.synchronize()
    finally:
        ver.destroy()


# ----------------------------------------------------------------------------- the step after: decode loop

def test_append_tokens_matches_oracle(jd):
    import torch
    from paper_2501_19309_amd import binding as jb
    rng = np.random.default_rng(0)
    for B, M, cap in ((1, 1, 4), (5, 7, 16), (64, 63, 130), (300, 10, 25)):
        buf = rng.integers(0, 1000, size=(B, cap)).astype(np.int32)
        lengths = rng.integers(0, cap + 1, size=B).astype(np.int32)
        draft = rng.integers(0, 128256, size=(B, M)).astype(np.int32)
        acc = rng.integers(0, M + 1, size=B).astype(np.int32)
        nxt = rng.integers(0, 128256, size=B).astype(np.int32)
        dbuf, dlen = torch.from_numpy(buf).cuda(), torch.from_numpy(lengths).cuda()
        rbuf, rlen = buf.copy(), lengths.astype(np.int64)
        for _ in range(3):   # several calls in a row, stream-ordered
            jb.append_tokens(torch.from_numpy(draft).cuda(), torch.from_numpy(acc).cuda(), torch.from_numpy(nxt).cuda(),
                             dbuf, dlen)
            vo.append_tokens(rbuf, rlen, draft, acc, nxt)
        torch.cuda.synchronize()
        assert np.array_equal(dbuf.cpu().numpy(), rbuf) and np.array_equal(dlen.cpu().numpy(), rlen), (B, M, cap)
    lib = jb.load_library()
    assert lib.jd_verify_append_tokens(1, 1, None, None, None, None, 4, None, None) == jb.JD_ERR_INVALID_ARG
    t = torch.zeros(8, dtype=torch.int32, device="cuda")
    p = t.data_ptr()
    assert lib.jd_verify_append_tokens(0, 1, p, p, p, p, 4, p, None) == jb.JD_ERR_SHAPE
    assert lib.jd_verify_append_tokens(1, 64, p, p, p, p, 4, p, None) == jb.JD_ERR_SHAPE
    assert lib.jd_verify_append_tokens(1, 1, p, p, p, p, 0, p, None) == jb.JD_ERR_SHAPE


@pytest.mark.parametrize("prenorm", [False, True], ids=["normalised", "prenorm"])
def test_decode_loop_token_buffers(jd, prenorm):
    # 12 iterations over 3 resident batches, one synchronisation at the end; the float64 oracle replays them
    import torch
    from paper_2501_19309_amd import decode_loop, harness
    shape = VerifyShape("loop", 6, 7, 256, 3000, "bf16", 1.0)
    host, dev = decode_loop.make_batches(shape, 3, 21, prenorm)
    assert all(np.array_equal(h["W"], host[0]["W"]) for h in host)
    assert not np.array_equal(host[0]["draft_tokens"], host[1]["draft_tokens"])
    ver = harness.make_verifier(dev[0])
    try:
        outs = [ver.alloc_outputs(shape.B, shape.M) for _ in range(3)]
        iters, cap = 12, 12 * (shape.M + 1)
        buf = torch.zeros(shape.B, cap, dtype=torch.int32, device="cuda")
        lengths = torch.zeros(shape.B, dtype=torch.int32, device="cuda")
        decode_loop.enqueue_loop(ver, dev, outs, buf, lengths, iters)
        torch.cuda.synchronize()
        gs = []
        for k in range(3):
            ref = prenorm_oracle(host[k]) if prenorm else oracle_for(host[k])
            gs.append(outs[k].to_numpy())
            compare(gs[k], ref)   # the last call on each batch, held to the oracle
        # The oracle's append step replays the loop.  It is fed the library's outputs, which compare() has just held
        # to the oracle (identical to the oracle's own unless a near-tie was decided the other way; every call on
        # one batch gives the same outputs).
        rbuf = np.zeros((shape.B, cap), dtype=np.int32); rlen = np.zeros(shape.B, dtype=np.int64)
        for i in range(iters):
            vo.append_tokens(rbuf, rlen, host[i % 3]["draft_tokens"], gs[i % 3]["accept_len"], gs[i % 3]["next_token"])
        assert np.array_equal(lengths.cpu().numpy(), rlen)
        assert np.array_equal(buf.cpu().numpy(), rbuf)
        assert rlen.min() >= iters and rlen.max() <= cap
    finally:
        ver.destroy()


FULL_SIZE = [(name, seed) for name in ("C2", "C3", "C4") for seed in (0, 1, 2)] + [("C4q", 0), ("C3q", 0), ("C4i", 0)]


@pytest.mark.parametrize("name,seed", FULL_SIZE, ids=lambda v: str(v))
def test_full_size_single_sequence(jd, name, seed):
    # full-size configs in the launch configuration the benchmark times; the oracle
    # evaluates the whole call (B = 1)
    print(f"[case] {name} seed {seed}", flush=True)
    x = make_inputs(CONFIGS[name], seed)
    print("[inputs ready]", flush=True)
    got = jd.run_once(x)
    print("[gpu done]", got["accept_len"], got["next_token"], flush=True)
    ref = oracle_for(x)
    rep = compare(got, ref)
    print(name, seed, rep, flush=True)


def test_full_size_prenorm_C4(jd):
    # the headline shape through the pre-norm entry point, as `bench.py --prenorm` times it
    print("[case] C4 prenorm", flush=True)
    x = make_inputs(CONFIGS["C4"], 0, prenorm=True)
    print("[inputs ready]", flush=True)
    got = jd.run_once(x)
    print("[gpu done]", got["accept_len"], got["next_token"], flush=True)
    rep = compare(got, prenorm_oracle(x))
    print("C4 prenorm", rep, flush=True)


@pytest.mark.parametrize("name,seed", [("C5", 0), ("C5", 1), ("C5q", 0), ("C5i", 0)], ids=lambda v: str(v))
def test_full_size_batched_sampled_sequences(jd, name, seed):
    # B = 64 sequences are independent, so the oracle checks a sample of them exactly: 16 sequences, eight in each
    # of the two 352-row tiles of the launch (sequences 0..31 and 32..63), first and last rows of both included
    print(f"[case] {name} seed {seed}", flush=True)
    cfg = CONFIGS[name]
    x = make_inputs(cfg, seed)
    print("[inputs ready]", flush=True)
    got = jd.run_once(x)
    print("[gpu done]", flush=True)
    seqs = [0, 3, 7, 12, 16, 21, 25, 31, 32, 35, 38, 44, 49, 54, 60, 63]
    ref = oracle_for(x, seqs=seqs)
    sub = {k: v[seqs] for k, v in got.items()}
    rep = compare(sub, ref)
    print(name, seed, rep, flush=True)
    # properties that hold for every sequence
    assert ((got["accept_len"] >= 0) & (got["accept_len"] <= cfg.M)).all()
    assert ((got["next_token"] >= 0) & (got["next_token"] < cfg.V)).all()
    assert (got["status"] == 0).all()
    z = (got["z_stand"] | got["z_judge"]).astype(bool)
    lead = np.argmin(np.concatenate([z, np.zeros((64, 1), bool)], 1), 1)
    assert np.array_equal(lead, got["accept_len"])
