"""The verification head in its calling pattern, and a batch-size sweep.

    python -m paper_2501_19309_amd.decode_loop --config C4 --iters 200
    python -m paper_2501_19309_amd.decode_loop --sweep 1,2,4,8,16,32,64,128

Speculative decoding repeats "draft M tokens, verify, add the accepted tokens and the one new token
to the context" (Sec. 3.1, paragraph after Eq. 4).  The draft model and the target trunk are not
part of this library, so the loop below stands in for them with pre-drawn synthetic batches that
are already resident in HBM: iteration i verifies batch i mod K (same weights, fresh embeddings,
draft tokens, draft logits and uniforms) and then appends to each sequence's token buffer with
``jd_verify_append_tokens``.  Everything is enqueued on one stream; the host synchronises once,
after the last iteration.  Reported: time per iteration against the time of the verify call alone
(what the appended step and the changing inputs cost), and tokens emitted per call.

``--sweep`` times the head at M = 10, d = 8192, V = 128256 (bf16) for a list of batch sizes:
the row count R = B (M + 1) crosses from the HBM-bound regime (W_lm streamed once, R <= 64 rows
per launch) into the MFMA-bound one.  One line of JSON per batch size.

Argument marshalling and timing only: every step of the path runs in the HIP library.  The token
buffers this loop produces are checked against a float64 replay in the GPU test-suite.
"""

from __future__ import annotations

import argparse
import json
import sys
import time
from typing import Dict, List


from . import binding as jb, harness


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def enqueue_loop(ver: "jb.JDVerify", batches: List[Dict], outs: List["jb.VerifyOutputs"], token_buf, lengths,
                 iters: int) -> None:
    """Enqueue `iters` verify + append steps on the current stream, cycling through `batches`
    (device-tensor dicts from harness.to_device).  No host synchronisation."""
    K = len(batches)
    for i in range(iters):
        s, o = batches[i % K], outs[i % K]
        if "hidden" in s:
            ver.run_prenorm(s["hidden"], s["gamma"], s["rms_eps"], s["draft_tokens"], s["draft_logits"], s["uniforms"], o)
        else:
            ver.run(s["emb"], s["draft_tokens"], s["draft_logits"], s["uniforms"], o)
        jb.append_tokens(s["draft_tokens"], o.accept_len, o.next_token, token_buf, lengths)


def make_batches(shape, n_sets: int, seed: int, prenorm: bool):
    """n_sets input batches for one model (weights of `seed`), numpy and device copies; W is uploaded once."""
    from synth import make_inputs

    host, dev = [], []
    for k in range(n_sets):
        x = make_inputs(shape, seed + k, prenorm=prenorm, weights_seed=seed)
        if k > 0:  # one model: share the weight tensors
            for name in ("W", "w_judge", "w_scale", "gamma"):
                if name in x:
                    x[name] = host[0][name]
        host.append(x)
        d = harness.to_device({n: v for n, v in x.items() if k == 0 or n not in ("W", "w_judge", "w_scale", "gamma")})
        if k > 0:
            for name in ("W", "w_judge", "w_scale", "gamma"):
                if name in dev[0]:
                    d[name] = dev[0][name]
        if prenorm:
            d["rms_eps"] = float(x["rms_eps"])
        dev.append(d)
    return host, dev


def loop_benchmark(config: str, iters: int, n_sets: int, seed: int, prenorm: bool, graph: bool = False) -> dict:
    import torch
    from synth import CONFIGS

    shape = CONFIGS[config]
    B, M = shape.B, shape.M
    t0 = time.time()
    host, dev = make_batches(shape, n_sets, seed, prenorm)
    log(f"[loop] {n_sets} batches of {shape.name} drawn in {time.time() - t0:.1f}s")
    ver = harness.make_verifier(dev[0])
    outs = [ver.alloc_outputs(B, M) for _ in range(n_sets)]
    cap = iters * (M + 1)
    token_buf = torch.zeros(B, cap, dtype=torch.int32, device="cuda")
    lengths = torch.zeros(B, dtype=torch.int32, device="cuda")

    def verify_only(n):
        for i in range(n):
            s, o = dev[i % n_sets], outs[i % n_sets]
            if prenorm:
                ver.run_prenorm(s["hidden"], s["gamma"], s["rms_eps"], s["draft_tokens"], s["draft_logits"], s["uniforms"], o)
            else:
                ver.run(s["emb"], s["draft_tokens"], s["draft_logits"], s["uniforms"], o)

    verify_only(20)
    torch.cuda.synchronize()
    t0 = time.perf_counter(); verify_only(iters); torch.cuda.synchronize()
    ms_verify = (time.perf_counter() - t0) * 1e3 / iters

    enqueue_loop(ver, dev, outs, token_buf, lengths, 20)
    torch.cuda.synchronize()
    token_buf.zero_(); lengths.zero_()
    torch.cuda.synchronize()
    t0 = time.perf_counter(); enqueue_loop(ver, dev, outs, token_buf, lengths, iters); torch.cuda.synchronize()
    ms_loop = (time.perf_counter() - t0) * 1e3 / iters

    L = lengths.cpu().numpy()
    rec = {
        "what": "decode loop: verify + append per iteration, one stream, one host synchronisation at the end",
        "workload": f"{shape.name}: B={B} M={M} d={shape.d} V={shape.V} {shape.dtype}, {n_sets} resident batches"
                    + (", pre-norm wiring" if prenorm else ""),
        "iters": iters, "ms_per_iteration": ms_loop, "ms_per_verify_call_alone": ms_verify,
        "append_and_rotation_overhead_us": (ms_loop - ms_verify) * 1e3,
        "tokens_per_sequence_per_call": float(L.mean()) / iters,
        "emitted_tokens_per_s": float(L.sum()) / (ms_loop * 1e-3 * iters),
        "verified_positions_per_s": B * M / (ms_loop * 1e-3),
    }
    if graph:
        # the same iterations as HIP graphs: one captured (verify + append) per resident batch, replayed in turn
        graphs = []
        for k in range(n_sets):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                enqueue_loop(ver, dev[k:k + 1], outs[k:k + 1], token_buf, lengths, 1)
            graphs.append(g)
        token_buf.zero_(); lengths.zero_()
        for i in range(20):
            graphs[i % n_sets].replay()
        torch.cuda.synchronize()
        token_buf.zero_(); lengths.zero_()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(iters):
            graphs[i % n_sets].replay()
        torch.cuda.synchronize()
        rec["ms_per_iteration_graph_replay"] = (time.perf_counter() - t0) * 1e3 / iters
        rec["graph_replay_same_lengths"] = bool((lengths.cpu().numpy() == L).all())
    ver.destroy()
    return rec


def sweep(batch_sizes: List[int], steps: int, seed: int, dtype: str = "bf16") -> List[dict]:
    import torch
    from synth import VerifyShape, make_inputs

    Bmax, M, d, V = max(batch_sizes), 10, 8192, 128256
    shape = VerifyShape("sweep", Bmax, M, d, V, dtype, (0.5, 2.5), "70B-shaped head, batch sweep")
    t0 = time.time()
    x = make_inputs(shape, seed)
    log(f"[sweep] inputs for B={Bmax} drawn in {time.time() - t0:.1f}s")
    dev = harness.to_device(x)
    ver = harness.make_verifier(dev)   # max_B = Bmax: one context, one re-tiled W_lm for every batch size
    recs = []
    w_bytes = V * d * (1 if dtype in ("fp8", "int8") else 2)
    for B in batch_sizes:
        R = B * (M + 1)
        e, t, D, u = (dev[k][:B].contiguous() for k in ("emb", "draft_tokens", "draft_logits", "uniforms"))
        out = ver.alloc_outputs(B, M)
        for _ in range(5):
            ver.run(e, t, D, u, out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            ver.run(e, t, D, u, out)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        ver.profile_begin(steps)
        for _ in range(steps):
            ver.run(e, t, D, u, out)
        torch.cuda.synchronize()
        kms, _ = ver.profile_end()
        lm = kms["lmhead"]
        kernel = "skinny (W_lm streamed once)" if R <= 64 else ("352-row kernel" if R > 176 else "176-row kernel")  # the library's dispatch
        recs.append({"B": B, "M": M, "W_lm": dtype, "rows": R, "ms_per_call": ms, "verified_positions_per_s": B * M / (ms * 1e-3),
                     "lmhead_ms": lm, "lmhead_kernel": kernel,
                     "lmhead_W_GBs": w_bytes / (lm * 1e-3) / 1e9, "lmhead_frac_hbm_peak": w_bytes / (lm * 1e-3) / 8e12,
                     "lmhead_TFLOPs": 2.0 * R * d * V / (lm * 1e-3) / 1e12,
                     "lmhead_frac_mfma_peak": 2.0 * R * d * V / (lm * 1e-3) / 2.5e15,
                     "other_kernels_ms": {k: v for k, v in kms.items() if k != "lmhead"}})
        log(f"[sweep] B={B:4d} R={R:5d} {ms:.4f} ms/call  lmhead {lm:.4f} ms ({kernel})")
    ver.destroy()
    return recs


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="C4")
    ap.add_argument("--iters", type=int, default=200)
    ap.add_argument("--sets", type=int, default=3, help="resident input batches the loop cycles through")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--prenorm", action="store_true")
    ap.add_argument("--graph", action="store_true", help="also time the loop as replayed HIP graphs")
    ap.add_argument("--sweep", default="", help="comma-separated batch sizes; runs the sweep instead of the loop")
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--dtype", default="bf16", choices=("bf16", "fp8", "int8"), help="W_lm storage type of the sweep")
    args = ap.parse_args()
    jb.load_library()
    if args.sweep:
        for rec in sweep([int(b) for b in args.sweep.split(",")], args.steps, args.seed, args.dtype):
            print(json.dumps(rec))
    else:
        print(json.dumps(loop_benchmark(args.config, args.iters, args.sets, args.seed, args.prenorm, args.graph)))
    return 0


if __name__ == "__main__":
    sys.exit(main())
