"""GPU test of jd_verify_run_noalloc, the entry point for callers that cannot allocate device memory: through
the C ABI, against jd_verify_run on a context (the same kernels: every output must be identical) and against the
float64 oracle, on two calls in a row, the second with a smaller input that lays the shared static workspace out
differently.  Collected last on purpose: it must pass in a fresh process and after every other GPU test."""

import numpy as np
import pytest

from oracle import verify_oracle as vo
from oracle.compare import compare
from synth import VerifyShape, make_inputs

pytestmark = pytest.mark.gpu


def _both_ways(x, shape, **cfg_kw):
    """(outputs of jd_verify_run_noalloc, outputs of jd_verify_run on a context) for one input dict."""
    import torch
    from paper_2501_19309_amd import binding as jb, harness
    dev = harness.to_device(x)
    cfg = jb.make_config(shape.d, shape.V, shape.B, shape.M, w_dtype=jb.JD_F32, **cfg_kw)
    out = jb.alloc_outputs(shape.B, shape.M, shape.V, want_probs=True)
    jb.run_noalloc(cfg, dev["W"], dev["w_judge"], dev["emb"], dev["draft_tokens"], dev["draft_logits"], dev["uniforms"], out)
    torch.cuda.synchronize()
    got = out.to_numpy()
    want = harness.run_once(x, want_probs=True, **cfg_kw)
    return got, want


def test_noalloc_matches_the_context_entry_point_and_the_oracle():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a HIP device"
    from paper_2501_19309_amd import binding as jb
    jb.load_library()
    # first call: ragged sizes, 99 rows; second call: fewer, shorter rows (every offset in the workspace moves);
    # third: the first again, so that it also runs on top of the second's leftovers
    big = VerifyShape("na_big", 9, 10, 100, 5000, "f32", 1.5)
    small = VerifyShape("na_small", 2, 4, 64, 777, "f32", 1.0)
    for shape, seed in ((big, 3), (small, 4), (big, 5)):
        print(f"[case] {shape.name} seed {seed}", flush=True)
        x = make_inputs(shape, seed)
        got, want = _both_ways(x, shape)
        for k in want:
            assert np.array_equal(got[k], want[k], equal_nan=True), (shape.name, k)
        ref = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"], return_probs=True)
        print(shape.name, compare(got, ref), flush=True)
    # the top-K rule uses one more array of the workspace
    x = make_inputs(small, 6)
    got, want = _both_ways(x, small, rule=jb.JD_RULE_TOPK, top_k=3)
    for k in want:
        assert np.array_equal(got[k], want[k], equal_nan=True), k
    ref = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"],
                    rule=vo.RULE_TOPK, top_k=3, return_probs=True)
    compare(got, ref, rule_topk=True)


def test_noalloc_rejects_what_it_cannot_hold():
    import torch
    from paper_2501_19309_amd import binding as jb
    jb.load_library()
    t = torch.zeros(64, dtype=torch.float32, device="cuda")
    p = t.data_ptr()
    outs = jb.alloc_outputs(1, 1)
    o = jb.outputs_struct(outs)
    ok = jb.make_config(8, 8, 1, 1, w_dtype=jb.JD_F32)
    call = lambda cfg, B=1, M=1, W=p, o=o: jb.run_noalloc_raw(cfg, W, p, B, M, p, None, p, p, M, p, o)
    # 27 rows of 128256 logits need 13.9 MB + partials: fits; 40 rows do not; nothing is launched for them
    fits = jb.make_config(16, 128256, 1, 26, w_dtype=jb.JD_F32)
    too_big = jb.make_config(16, 128256, 1, 39, w_dtype=jb.JD_F32)
    assert 27 * 128256 * 4 < jb.JD_NOALLOC_SCRATCH_BYTES < 40 * 128256 * 4
    assert call(too_big, 1, 39) == jb.JD_ERR_SHAPE
    assert b"needs" in jb.load_library().jd_verify_last_error_detail()
    assert call(jb.make_config(8, 8, 1, 1, w_dtype=jb.JD_BF16)) == jb.JD_ERR_UNSUPPORTED_DTYPE
    assert call(ok, W=None) == jb.JD_ERR_INVALID_ARG
    assert call(ok, o=None) == jb.JD_ERR_INVALID_ARG
    assert call(ok, B=2) == jb.JD_ERR_SHAPE
    assert call(jb.make_config(8, 8, 1, 1, w_dtype=jb.JD_F32, delta=0.3)) == jb.JD_ERR_INVALID_ARG
    assert call(jb.make_config(8, 8, 1, 1, w_dtype=jb.JD_F32, device=1)) in (jb.JD_ERR_INVALID_ARG, jb.JD_ERR_HIP)
    del fits
    torch.cuda.synchronize()


def test_noalloc_under_graph_capture():
    # what the entry point is for: captured into a HIP graph (no allocation, no synchronisation, no memset node) and
    # replayed with fresh inputs, eager work and synchronisations between the replays; every replay must equal the
    # eager result and satisfy the parity bar against the oracle
    import torch
    from paper_2501_19309_amd import binding as jb, harness
    jb.load_library()
    shape = VerifyShape("na_graph", 4, 6, 96, 1500, "f32", 1.2)
    xs = [make_inputs(shape, 50 + k, weights_seed=50) for k in range(2)]
    dev = harness.to_device(xs[0])
    cfg = jb.make_config(shape.d, shape.V, shape.B, shape.M, w_dtype=jb.JD_F32)
    out = jb.alloc_outputs(shape.B, shape.M, shape.V)

    def call():
        jb.run_noalloc(cfg, dev["W"], dev["w_judge"], dev["emb"], dev["draft_tokens"], dev["draft_logits"], dev["uniforms"], out)

    call()   # eager once: also the first call on the device, which looks up the workspace's address
    torch.cuda.synchronize()
    eager0 = out.to_numpy()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for it, k in enumerate((1, 0, 1)):
        x = xs[k]
        fresh = harness.to_device({n: x[n] for n in ("emb", "draft_tokens", "draft_logits", "uniforms")})
        for n, t in fresh.items():
            dev[n].copy_(t)      # eager work between the replays
        for t in (out.accept_len, out.next_token, out.status):
            t.fill_(-7)          # a replay that did nothing would be noticed
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = out.to_numpy()
        ref = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"])
        print("replay", it, compare(got, ref), flush=True)
        if k == 0:
            for name, v in got.items():
                assert np.array_equal(v, eager0[name], equal_nan=True), (it, name)


def test_noalloc_from_a_plain_cpp_process(tmp_path):
    # the same entry point called from tests/cabi_check.cpp: a process with the HIP runtime and this library only
    # (no torch, no context ever created), so the look-up of the static workspace happens on its very first call
    import os
    import subprocess
    from paper_2501_19309_amd import binding as jb
    from paper_2501_19309_amd.build import CABI_CHECK_PATH
    assert os.path.exists(CABI_CHECK_PATH), "jd_cabi_check is not built: run __graft_entry__.build()"
    shape = VerifyShape("na_cpp", 3, 6, 72, 1030, "f32", 1.0)
    x = make_inputs(shape, 8)
    for name in ("emb", "W", "w_judge", "draft_logits", "draft_tokens", "uniforms"):
        np.ascontiguousarray(x[name]).tofile(tmp_path / f"{name}.bin")
    cmd = [CABI_CHECK_PATH, str(tmp_path), str(shape.B), str(shape.M), str(shape.d), str(shape.V), str(jb.JD_F32), "2"]
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
    ref = vo.verify(x["emb"], x["W"], x["w_judge"], x["draft_tokens"], x["draft_logits"], x["uniforms"])
    print(compare(got, ref), flush=True)
