#!/usr/bin/env python3
"""Benchmark of the verify -> accept -> commit -> retrieve step on one MI355X.

A "step" is one pass of the whole hot path for one batch of synthetic input:
dbl_retrieve -> dbl_build_window -> dbl_verify_block -> dbl_accept -> dbl_kv_commit,
chained on the device with no host decision in between.  Default workload: the
LLaMA-3.3-70B-shaped bf16 target (80 layers, d 8192, 64/8 heads, FFN 28672, vocab
128256; random weights from a seed, resident in HBM), a 2048-token KV cache built by
real prefill of a Zipf(1.1) token stream with 20% repeated 16-grams, window k = 8,
batch 1, greedy acceptance.

Prints ONE JSON line: metric/value/unit (verified window positions per second), ms_per_step (wall
clock over the K timed steps), ms_per_step_median (median of per-step HIP-event times on the context's
stream), hbm_GBps_step (algorithmic bytes of a step / step time), breakdown_ms (per call, from events on
the context's stream), projections (each projection kernel timed alone), roofline (the dominant
kernel, fused gate/up: achieved GB/s from live HIP-event timing; HBM traffic as recorded by rocprofv3 for
exactly the launch shape the library reports, else null) and cpu_baseline (the CPU oracle timed on this
host).  `--also w1,w2` appends the same summary for further workloads under "other_workloads".
`--gpus N` with N > 1 is not supported: this build runs on one GPU.  `--double` measures the two-model
Double round instead.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E peak
# HBM bytes one launch of the dominant kernel (fused gate/up projection: gemm_rows_kernel plus
# the xn_kernel that stores its normalised input) moves, from two rocprofv3 --pmc runs
# (FETCH_SIZE scaled by 2.000, the factor a plain 1 GiB copy gives on this machine, plus
# WRITE_SIZE); summary in profiles/gate_up_projection_llama70b_traffic.txt.
# Counters cannot be read inside this process, so the figure is the recorded one; it is reported only while
# the library still launches the gate/up projection the way it did under the profiler (dbl_projection_plan:
# kernel form, tile rows per unit, workgroups, split units), else null.
MEASURED_TRAFFIC = {"llama70b_ctx2048_k8_b1_greedy": {"bytes": 944_430_490,          # (460 158.4 + 300.0) KiB x 2.000 + 875.7 + 502.9 KiB
                                                      "plan": (1, 2, 256, 0),        # gemm_rows_kernel, Q = 2, 256 workgroups, whole units
                                                      "kernel": "gemm_rows_kernel<bf16, EPI_SWIGLU, R=1, Q=2> after xn_kernel"}}

WORKLOADS = {
    # name: (shape key, context, k, batch, mode, temperature, repeat fraction, span lo, span hi)
    "llama70b_ctx2048_k8_b1_greedy": ("llama70b", 2048, 8, 1, "greedy", 0.0, 0.20, 16, 16),
    "llama1b_ctx1024_k8_b1_greedy": ("llama1b", 1024, 8, 1, "greedy", 0.0, 0.15, 16, 16),
    "qwen32b_ctx8192_k16_b1_sample": ("qwen32b", 8192, 16, 1, "sample", 0.7, 0.20, 16, 16),
    "tiny_ctx256_k4_b1_greedy": ("tiny", 256, 4, 1, "greedy", 0.0, 0.25, 8, 8),
    # higher concurrency (App. D.1's regime): 64 and 128 window rows per step at the headline context
    "llama70b_ctx2048_k8_b8_greedy": ("llama70b", 2048, 8, 8, "greedy", 0.0, 0.20, 16, 16),
    "llama70b_ctx2048_k8_b16_greedy": ("llama70b", 2048, 8, 16, "greedy", 0.0, 0.20, 16, 16),
    # long-context stress: the KV cache is a seeded fill (dbl_kv_fill), not a prefill: bandwidth runs
    "llama70b_ctx32768_k4_b4_sample": ("llama70b", 32768, 4, 4, "sample", 1.0, 0.30, 8, 64),
    "llama70b_ctx32768_k8_b4_sample": ("llama70b", 32768, 8, 4, "sample", 1.0, 0.30, 8, 64),
    "llama70b_ctx32768_k16_b4_sample": ("llama70b", 32768, 16, 4, "sample", 1.0, 0.30, 8, 64),
    "llama70b_ctx32768_k32_b4_sample": ("llama70b", 32768, 32, 4, "sample", 1.0, 0.30, 8, 64),
}


# the other named configurations, summarised beside the headline line by default (they add about a minute)
DEFAULT_ALSO = "llama1b_ctx1024_k8_b1_greedy,qwen32b_ctx8192_k16_b1_sample,llama70b_ctx32768_k32_b4_sample"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(shape_key: str, k: int, ctx: int, full_layers: int, full_vocab: int, budget_s: float = 12.0):
    """The oracle, as it stands, timed on this host's cores on a bounded sample: two full-width decoder
    layers plus a 1/8-vocabulary LM-head slice over k window rows behind a context of `ctx` cached tokens
    (seeded keys and values written into the oracle's cache: a prefill of that length at full width would
    take the oracle minutes), repeated until about `budget_s` seconds of CPU work have been timed; the full
    step is extrapolated as layers * t_layer + 8 * t_lm_slice."""
    import numpy as np
    import oracle as O
    from paper_2601_05524_amd import synth
    shape = dict(synth.CONFIGS[shape_key])
    small = shape["d_model"] <= 2048
    vdiv = 1 if small else 8
    nl_sample = min(2, max(1, full_layers))
    vs = shape["vocab"] // vdiv
    ctx = min(ctx, 4096)                      # (the oracle's attention is one core's work: bounded)
    shape.update(vocab=vs, max_ctx=ctx + 64)
    cores = len(os.sched_getaffinity(0))
    win = (np.arange(k, dtype=np.int32) * 7919 + 13) % vs
    times, reps = {}, {}
    for nl in (0, nl_sample):
        m = O.Model(**dict(shape, n_layers=nl), seed=synth.BASE_SEED)
        s = O.Seq(m, max_hist=64)
        if nl > 0 and ctx > 0:
            rng = np.random.default_rng(1)
            s.kcache()[:, :, :ctx, :] = rng.standard_normal((nl, shape["n_kv_heads"], ctx, shape["head_dim"])).astype(np.float32)
            s.vcache()[:, :, :ctx, :] = rng.standard_normal((nl, shape["n_kv_heads"], ctx, shape["head_dim"])).astype(np.float32)
        share = budget_s * (0.1 if nl == 0 else 0.9)
        n, t0 = 0, time.perf_counter()
        while True:
            s.reset()
            if nl > 0 and ctx > 0:
                s.commit(ctx, [])             # the planted rows count as committed
            s.verify_block(win)
            n += 1
            if time.perf_counter() - t0 >= share or n >= 200:
                break
        times[nl] = (time.perf_counter() - t0) / n
        reps[nl] = n
        s.close(); m.close()
    t_lm = times[0]
    t_layer = max(times[nl_sample] - times[0], 1e-9) / nl_sample
    t_full = full_layers * t_layer + vdiv * t_lm
    return {"value": k / t_full, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": "%d full-width layers + 1/%d-vocab LM head, k=%d rows behind %d cached tokens (seeded K/V), "
                      "%d + %d repetitions (%.1f s of CPU work); extrapolated to %d layers + full vocab "
                      "(t_layer=%.3fs, t_lm_slice=%.3fs)"
                      % (nl_sample, vdiv, k, ctx, reps[nl_sample], reps[0],
                         times[0] * reps[0] + times[nl_sample] * reps[nl_sample], full_layers, t_layer, t_lm),
            "extrapolated": True}


def bench_double(args):
    """Not the headline line: the full Double round (two models, two streams) against plain
    greedy decoding and against target-only retrieval decoding on the same kernels.
    70B-shaped target + 1B-shaped draft, both bf16 with random weights from a seed, so the
    draft's proposals are unrelated to the target: this measures the machinery's cost and the
    contention of draft-when-verify on ONE device, not an acceptance rate."""
    import math
    import numpy as np
    import torch
    from paper_2601_05524_amd import binding as B
    from paper_2601_05524_amd import double_round as DR
    from paper_2601_05524_amd import synth

    torch.cuda.set_device(0)
    P, k_p, k_q, n_new = 2048, 8, 8, args.double_tokens
    tshape, dshape = dict(synth.CONFIGS["llama70b"]), dict(synth.CONFIGS["llama1b"])
    if args.layers > 0:
        tshape["n_layers"] = args.layers
    room = P + 64 * (n_new + 64)
    kw = dict(max_ctx=((P + 24 * (n_new + 64)) // 64 + 1) * 64, max_window=16, max_hist=room)
    target = DR.Lane(tshape, synth.BASE_SEED + 2, **kw)
    draft = DR.Lane(dshape, synth.BASE_SEED + 1, **kw)
    prompt = [int(t) for t in synth.zipf_history(synth.BASE_SEED + 2, P + 1, tshape["vocab"], 1.1, 0.20, 16, 16)]

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps

    target.load(prompt)
    draft.load(prompt)
    torch.cuda.synchronize()
    # T_p: one target Retrieval Forward; T_q: one draft Retrieval Forward; gamma = ceil(T_p / T_q)
    T_p = timed(lambda: target.chain(1, k_p), 5)
    T_q = timed(lambda: draft.chain(1, k_q), 20)
    gamma = max(1, min(args.double_gamma if args.double_gamma > 0 else math.ceil(T_p / T_q), 32))

    res = {}
    # the iterative retrieval drafter alone (Eq. 5): gamma chained Retrieval Forwards of the draft
    draft.load(prompt)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    draft.chain(gamma, k_q)
    chain = draft.generated()
    t_chain = time.perf_counter() - t0
    res["draft_chain"] = {"forwards": gamma, "L_draft": len(chain), "AMT": round(len(chain) / gamma - 1.0, 3),
                          "ms": round(t_chain * 1e3, 3), "ms_per_forward": round(t_chain / gamma * 1e3, 3)}
    # plain greedy decoding of the target, one token per forward
    target.load(prompt)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    DR.autoregressive_steps(target, min(n_new, 24))
    ar = target.generated()
    res["autoregressive"] = {"tokens": len(ar), "tokens_per_s": round(len(ar) / (time.perf_counter() - t0), 2)}
    # target-only retrieval decoding (the headline step, chained on the device)
    target.load(prompt)
    torch.cuda.synchronize()
    steps = max(8, n_new // 2)
    t0 = time.perf_counter()
    target.chain(steps, k_p)
    sd = target.generated()
    res["target_retrieval_only"] = {"tokens": len(sd), "forwards": steps,
                                    "tokens_per_s": round(len(sd) / (time.perf_counter() - t0), 2)}
    # the full Double round
    dec = DR.DoubleDecoder(target, draft, gamma=gamma, k_p=k_p, k_q=k_q)
    dec.start(prompt)
    t0 = time.perf_counter()
    while dec.emitted < n_new:
        dec.round()
    out, rounds = target.generated(), dec.rounds
    dt = time.perf_counter() - t0
    res["double"] = {"tokens": len(out), "rounds": len(rounds), "tokens_per_s": round(len(out) / dt, 2),
                     "ms_per_round": round(dt / len(rounds) * 1e3, 3),
                     "post_verify_rounds": sum(r["mode"] == "post" for r in rounds),
                     "drafted_per_round": round(sum(r["drafted"] for r in rounds) / len(rounds), 2)}
    same = 0
    while same < min(len(out), len(sd)) and out[same] == sd[same]:
        same += 1
    out_line = {
        "metric": "emitted tokens/s of a full Double round (70B-shaped target + 1B-shaped draft on two streams, greedy)",
        "value": res["double"]["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "higher_is_better": True,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "double_llama70b_llama1b_ctx2048_greedy", "k_target": k_p, "k_draft": k_q,
                   "gamma": gamma, "new_tokens": n_new, "target_layers": tshape["n_layers"]},
        "T_p_ms": round(T_p * 1e3, 3), "T_q_ms": round(T_q * 1e3, 3), "speed_ratio_C": round(T_p / T_q, 2),
        "results": res,
        "double_vs_autoregressive": round(res["double"]["tokens_per_s"] / res["autoregressive"]["tokens_per_s"], 3),
        "double_vs_target_retrieval_only": round(res["double"]["tokens_per_s"] / res["target_retrieval_only"]["tokens_per_s"], 3),
        "tokens_identical_to_target_retrieval_only": same == min(len(out), len(sd)),
        "note": "random weights: the draft model's proposals are unrelated to the target's, so drafts are rejected; "
                "the paper's 5.3x / 2.8x are for trained model pairs on separate A100s (context, not comparable)",
    }
    target.close(); draft.close()
    print(json.dumps(out_line), flush=True)


def run_workload(args, workload, with_cpu_baseline):
    """One workload: create the model, build the context, time K steps.  Returns the JSON object."""
    import numpy as np
    import torch
    from paper_2601_05524_amd import binding as B
    from paper_2601_05524_amd import synth

    shape_key, P, k, Bn, mode, T, frac, slo, shi = WORKLOADS[workload]
    shape = dict(synth.CONFIGS[shape_key])
    if args.layers > 0:
        shape["n_layers"] = args.layers
    idx = list(synth.CONFIGS).index(shape_key)
    seed = synth.BASE_SEED + idx
    steps, warm = args.steps, args.warmup
    chunk = min(16, 128 // Bn)      # rows of one prefill call stay within the library's 128
    if P > 8192:
        steps, warm = min(steps, 6), min(warm, 1)       # a 128-row window streams the weights 8 times
    max_ctx = ((P + (steps + warm + 6) * k + 63) // 64 + 1) * 64
    if args.paged_kv:
        max_ctx = (max_ctx + 255) // 256 * 256
    max_hist = P + 1 + (steps + warm + 6) * k + 64
    torch.cuda.set_device(0)
    dev = "cuda:0"
    t0 = time.perf_counter()
    cfg = B.make_cfg(**shape, max_batch=Bn, max_ctx=max_ctx, max_window=max(chunk, k), max_hist=max_hist,
                     flags=B.DBL_FLAG_PAGED_KV if args.paged_kv else 0)
    ctx = B.dbl_create(cfg, seed, torch.cuda.current_stream().cuda_stream)
    if args.tune:
        B.dbl_set_tuning(ctx, **dict((kv.split("=")[0], int(kv.split("=")[1])) for kv in args.tune.split(",")))
    wbytes, kv_per_tok = B.dbl_model_bytes(ctx)
    log("[bench] %s: context created in %.1fs: %.2f GB of weights streamed per step" % (workload, time.perf_counter() - t0, wbytes / 1e9))

    # history = P + 1 tokens; prefill the first P through verify_block + kv_commit
    prompts = [synth.zipf_history(seed + 100 * b, P + 1, shape["vocab"], 1.1, frac, slo, shi) for b in range(Bn)]
    for b, p in enumerate(prompts):
        B.dbl_history_set(ctx, b, np.ascontiguousarray(p, dtype=np.int32))
    keep = torch.empty(Bn, dtype=torch.int32, device=dev)
    t0 = time.perf_counter()
    filled = P > 8192      # too long to prefill in a benchmark: seeded stand-in K/V rows
    if filled:
        for b in range(Bn):
            B.dbl_kv_fill(ctx, b, P, seed + b)
    i = P if filled else 0
    while i < P:
        c = min(chunk, P - i)
        w = torch.as_tensor(np.stack([p[i:i + c] for p in prompts]).astype(np.int32), device=dev)
        keep.fill_(c)
        B.dbl_verify_block(ctx, w, Bn, c)
        B.dbl_kv_commit(ctx, keep)
        i += c
    torch.cuda.synchronize()
    kv0 = np.zeros(Bn, np.int32)
    B.dbl_kv_len(ctx, kv0)
    log("[bench] %s of %d tokens in %.1fs, kv_len=%s" % ("seeded KV fill" if filled else "prefill", P, time.perf_counter() - t0,
                                                         kv0.tolist()))

    max_cont = k - 1 if k > 1 else 1
    cont = torch.empty((Bn, max_cont), dtype=torch.int32, device=dev)
    cl, mn, mp = (torch.empty(Bn, dtype=torch.int32, device=dev) for _ in range(3))
    window = torch.empty((Bn, k), dtype=torch.int32, device=dev)
    n_acc = torch.empty(Bn, dtype=torch.int32, device=dev)
    emit = torch.empty((Bn, k), dtype=torch.int32, device=dev)
    guide = torch.empty((Bn, k), dtype=torch.int32, device=dev)
    amode = B.DBL_SAMPLE if mode == "sample" else B.DBL_GREEDY

    def step(i):
        B.dbl_retrieve(ctx, Bn, 3, 1, max_cont, cont, cl, mn, mp)
        B.dbl_build_window(ctx, Bn, k, max_cont, cont, cl, 0, window)
        B.dbl_verify_block(ctx, window, Bn, k, T, seed, i)
        B.dbl_accept(ctx, amode, None, n_acc, emit, guide)
        B.dbl_kv_commit(ctx, None)

    for i in range(warm):
        step(i)
    B.dbl_kv_len(ctx, kv0)          # synchronises
    # K steps between two synchronisations (wall clock), with an event between consecutive steps on the
    # context's stream (= torch's current stream) for the per-step times
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        step(warm + i)
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    ms_median = per_step[steps // 2] if steps % 2 else 0.5 * (per_step[steps // 2 - 1] + per_step[steps // 2])
    kv1 = np.zeros(Bn, np.int32)
    B.dbl_kv_len(ctx, kv1)
    emitted = int((kv1 - kv0).sum())      # sum over steps of n_acc + 1
    ms_step = dt / steps * 1e3
    ctx_mid = float(kv0.mean() + kv1.mean()) / 2 + k
    step_bytes = wbytes + Bn * ctx_mid * kv_per_tok
    step_gbps = step_bytes / (dt / steps) / 1e9

    # per-call breakdown (events on the context's stream = torch's current stream)
    names = ["retrieve", "build_window", "verify_block", "accept", "kv_commit"]
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
    acc = [0.0] * 5
    reps = 3
    for r in range(reps):
        ev[0].record()
        B.dbl_retrieve(ctx, Bn, 3, 1, max_cont, cont, cl, mn, mp); ev[1].record()
        B.dbl_build_window(ctx, Bn, k, max_cont, cont, cl, 0, window); ev[2].record()
        B.dbl_verify_block(ctx, window, Bn, k, T, seed, steps + warm + r); ev[3].record()
        B.dbl_accept(ctx, amode, None, n_acc, emit, guide); ev[4].record()
        B.dbl_kv_commit(ctx, None); ev[5].record()
        torch.cuda.synchronize()
        for j in range(5):
            acc[j] += ev[j].elapsed_time(ev[j + 1]) / reps
    breakdown = {n: round(v, 4) for n, v in zip(names, acc)}

    # dominant kernel: the fused gate/up + SwiGLU projection (55% of the bytes at 70B shape)
    M = min(128, Bn * k)   # rows of one projection pass (the LM head splits it into passes of 64)
    proj = {}
    for which, name in enumerate(["qkv", "o_proj", "gate_up_swiglu", "down_proj", "lm_head_stats"]):
        if which < 4 and shape["n_layers"] < 1:
            continue
        ms, nbytes = B.dbl_bench_projection(ctx, which, M, args.kernel_iters if which != 4 else max(4, args.kernel_iters // 4))
        proj[name] = {"ms": round(ms, 5), "GB/s": round(nbytes / ms / 1e6, 1), "bytes": nbytes}
    dom_which = 2 if "gate_up_swiglu" in proj else 4
    dom = proj.get("gate_up_swiglu") or proj["lm_head_stats"]
    plan = B.dbl_projection_plan(ctx, dom_which, M)
    forms = {0: "gemm_stream_kernel", 1: "gemm_rows_kernel", 2: "gemm_wide_swiglu_kernel", 3: "gemm_wide_slice_kernel + resid_reduce_kernel"}
    roofline = {"bound": "hbm",
                "kernel": "%s after xn_kernel (%s of one layer)" % (forms[plan[0]], "fused gate/up projection" if dom_which == 2 else "LM head"),
                "launch": {"tile_rows_per_unit": plan[1], "workgroups": plan[2], "split_units": bool(plan[3]), "rows": M},
                "achieved": dom["GB/s"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(dom["GB/s"] / HBM_PEAK_GBPS, 4), "traffic": None,
                "bytes_per_launch": dom["bytes"], "ms_per_launch": dom["ms"]}
    rec = MEASURED_TRAFFIC.get(workload)
    if rec and args.layers <= 0 and dom_which == 2 and tuple(plan) == rec["plan"] and not args.tune:
        roofline["traffic"] = rec["bytes"]
        roofline["traffic_unit"] = "bytes per launch (rocprofv3 FETCH_SIZE x 2.000 + WRITE_SIZE of %s, recorded in profiles/)" % rec["kernel"]
        roofline["traffic_vs_algorithmic"] = round(rec["bytes"] / dom["bytes"], 4)
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)     # 1 GiB
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    B.dbl_destroy(ctx)

    name = workload if args.layers <= 0 else "%s_first%dlayers" % (workload, args.layers)
    out = {
        "metric": "verified tokens/s of target verify step (70B-shape, k=8) + achieved HBM GB/s",
        "value": round(Bn * k / (dt / steps), 2), "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warm,
        "ms_per_step": round(ms_step, 4), "ms_per_step_median": round(ms_median, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if shape["dtype"] == 1 else "f32", "data": "synthetic",
        "config": {"workload": name, "ctx": P, "k": k, "batch": Bn,
                   "accept": mode, "weights": "random N(0,0.02) from seed %d" % seed,
                   "kv_cache": ("seeded fill" if filled else "prefill of the history") + (", paged" if args.paged_kv else "")},
        "hbm_GBps_step": round(step_gbps, 1), "hbm_frac_step": round(step_gbps / HBM_PEAK_GBPS, 4),
        "algorithmic_bytes_per_step": int(step_bytes), "emitted_tokens_per_s": round(emitted / dt, 2),
        "breakdown_ms": breakdown, "projections": proj, "roofline": roofline,
    }
    if with_cpu_baseline:
        t0 = time.perf_counter()
        full_layers = synth.CONFIGS[shape_key]["n_layers"] if args.layers <= 0 else args.layers
        out["cpu_baseline"] = cpu_baseline(shape_key, k, P, full_layers, shape["vocab"])
        log("[bench] oracle baseline took %.1fs" % (time.perf_counter() - t0))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama70b_ctx2048_k8_b1_greedy", choices=sorted(WORKLOADS))
    ap.add_argument("--also", default=DEFAULT_ALSO,
                    help="comma-separated further workloads, summarised under other_workloads ('' or 'none': only --workload)")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (0 = the model's own)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-iters", type=int, default=40, help="launches per projection for the roofline line")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference dispatch for scaling rocprofv3 --pmc byte counters)")
    ap.add_argument("--paged-kv", action="store_true", help="KV cache as a pool of 256-token pages (default: contiguous)")
    ap.add_argument("--tune", default="", help="dbl_tuning fields, e.g. attn_p16=0,split_units=-1 (measurement of kernel forms)")
    ap.add_argument("--double", action="store_true",
                    help="measure the full Double round (draft + target on two streams) instead of the headline step")
    ap.add_argument("--double-tokens", type=int, default=64)
    ap.add_argument("--double-gamma", type=int, default=0, help="draft iterations per round (0 = ceil(T_p / T_q))")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported" % args.gpus)
        sys.exit(2)

    if args.double:
        return bench_double(args)

    out = run_workload(args, args.workload, not args.no_cpu_baseline)
    others = [w for w in args.also.split(",") if w and w != "none" and w != args.workload]
    for w in others:
        if w not in WORKLOADS:
            log("bench.py: unknown workload %s" % w)
            sys.exit(2)
        o = run_workload(args, w, False)
        out.setdefault("other_workloads", {})[w] = {
            "ms_per_step": o["ms_per_step"], "ms_per_step_median": o["ms_per_step_median"], "value": o["value"], "unit": o["unit"],
            "hbm_GBps_step": o["hbm_GBps_step"], "hbm_frac_step": o["hbm_frac_step"], "steps": o["steps"],
            "roofline": {kk: o["roofline"][kk] for kk in ("kernel", "achieved", "frac", "ms_per_launch")}}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
