#!/usr/bin/env python3
"""Benchmark of the unified-KV decode hot path on one MI355X.

A step is one pass of the whole path over one mixed-service batch: grow every request by one
token (host: page allocation from the library's free list), then `ukv_plan_step`: the new
page-table entries, the store of every request's new K/V token into its pages and split-KV
decode attention with the merge of cut requests, as ONE launch of a plan that is kept across
steps (remade every 64 tokens of growth).  `--replan-each-step` plans and uploads in every step
(`ukv_decode_step`: plan upload + decode launch); `--separate-append` runs the step as
`ukv_append` + `ukv_decode_attention`.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

  value      whole-step KV throughput: sum over steps of ctx_len*token_bytes / wall time
  roofline   the decode kernel alone: algorithmic KV bytes per launch / its mean duration,
             measured with HIP events on the launch stream inside the timed region
  cpu_baseline  the fp64 oracle timed on the host cores on a bounded sample of the same batch
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E
WORKLOAD_NAMES = {
    1: "cfg1: one service 8/8 heads d=64, 8 requests, ctx U[64,512]",
    2: "cfg2: Llama-2-7B-shaped layer 32/32 d=128, 64 requests, ctx U[128,4096], 4 GiB pool",
    3: "cfg3: two services (32/32 d=128 + 40/40 d=128) sharing one pool, 128 requests, "
       "ctx lognormal(median 1024, max 8192), 16 KiB pages interleaved, 4 GiB pool",
    4: "cfg4: GQA mix (32/8 + 64/8, d=128), 256 requests, ctx lognormal(median 2048, max 32768), "
       "churned 4 GiB pool",
    5: "cfg5: four services (12/12 d=64, 32/32, 40/40, 32/8 d=128), 512 requests, "
       "ctx lognormal(median 1024, max 16384), churned 8 GiB pool",
}


def read_traffic(cfg: int):
    """HBM bytes per decode launch as the hardware counters gave them.  They cannot be read inside this run (they
    need two rocprofv3 --pmc passes), so they come from the committed summary of such passes over this command,
    together with the algorithmic bytes of THAT run (a few steps earlier in the same batch's life, so a fraction of
    a per cent smaller than this run's) and their ratio: (traffic, source) or (None, None)."""
    name = f"decode_kernel_cfg{cfg}_pmc.txt"
    try:
        text = open(os.path.join(ROOT, "profiles", name)).read()
        get = lambda key: float(re.search(rf"^{key}:\s*([0-9.eE+]+)", text, re.M).group(1))
        return get("traffic_bytes_per_launch"), {
            "file": "profiles/" + name, "algorithmic_bytes_per_launch_in_that_run": int(get("algorithmic_bytes_per_launch")),
            "traffic_over_algorithmic": get("traffic_over_algorithmic")}
    except (OSError, AttributeError):
        return None, None


def cpu_baseline(batch, kv_bytes_total: int, target_s: float = 15.0, one_thread: bool = False):
    """Time the oracle (attention) on a bounded sample of the batch's requests."""
    import numpy as np
    from oracle import oracle
    n = batch.n_requests
    order = np.random.default_rng(0).permutation(n)
    tb = batch.token_bytes()
    probe = order[:min(n, 8)]
    t0 = time.perf_counter()
    oracle.attention(batch, batch.pool, requests=probe)
    dt = time.perf_counter() - t0
    probe_bytes = int((batch.ctx_len[probe].astype(np.int64) * tb[probe]).sum())
    rate = probe_bytes / max(dt, 1e-9)
    want = rate * target_s
    csum = np.cumsum(batch.ctx_len[order].astype(np.int64) * tb[order])
    k = int(np.searchsorted(csum, want)) + 1
    sample = order[:min(n, max(k, len(probe)))]
    t0 = time.perf_counter()
    oracle.attention(batch, batch.pool, requests=sample)
    dt = time.perf_counter() - t0
    sb = int((batch.ctx_len[sample].astype(np.int64) * tb[sample]).sum())
    cores = oracle.threads()
    res = {
        "value": sb / dt / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
        "sample": f"{len(sample)} of {n} requests of the same batch ({sb / 1e9:.3f} GB of KV, one attention "
                  f"step, {dt:.1f} s, fp64, OpenMP over requests)",
        "tokens_per_s": len(sample) / dt,
    }
    if one_thread:  # the small workloads also on a single core
        t0 = time.perf_counter()
        oracle.attention(batch, batch.pool, requests=sample, n_threads=1)
        dt1 = time.perf_counter() - t0
        oracle.attention(batch, batch.pool, requests=probe[:1], n_threads=cores)  # back to all cores
        res["one_thread"] = {"value": round(sb / dt1 / 1e9, 4), "unit": "GB/s", "cores": 1, "seconds": round(dt1, 2)}
    return res


MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16

PREFILL_WORKLOADS = {
    # name: (service shapes, request mix, prompt-length law, n prompts, pool pages)
    "chat": (("7b", "8b"), (0.5, 0.5), dict(kind="lognormal", median=1024, sigma=0.8, max=8192), 32, 1 << 17),
    "summarize": (("7b", "70b"), (0.5, 0.5), dict(kind="lognormal", median=13000, sigma=0.25, max=20000), 6,
                  1 << 17),
    # the head_dim 64 instantiation of the kernel (the 12-head service of the four-service workload)
    "small-heads": (("h12",), (1.0,), dict(kind="lognormal", median=4096, sigma=0.4, max=8192), 24, 1 << 17),
}


def main_prefill(args):
    """Prefill attention (next row after the decode path): whole prompts, causal; one JSON line."""
    import numpy as np
    import torch
    import paper_2504_15720_amd as U
    from synth import SHAPES, draw_prefill_inputs, make_batch
    from synth.workloads import draw_lengths
    from paper_2504_15720_amd.device_batch import DeviceBatch

    names, mix, law, n, pages = PREFILL_WORKLOADS[args.prefill_workload]
    rng = np.random.default_rng(20250415 + 77)
    services = [SHAPES[x] for x in names]
    sid = rng.choice(len(services), size=n, p=mix)
    ctx = np.maximum(draw_lengths(law, n, rng), 64)
    b = make_batch(services, sid, ctx, pages, "permutation", rng, pool_seed=11)
    db = DeviceBatch(b, profile=True)
    if args.prefill_no_xcd:
        U.ukv_set_param(db.pool, U.UKV_PARAM_PREFILL_XCD, 0)
    U.ukv_set_param(db.pool, U.UKV_PARAM_PREFILL_WEIGHTS, args.prefill_weights)
    q_bits, q_off, out_off, n_el = draw_prefill_inputs(b, ctx, rng)
    _, run = db.prefill(ctx, q_bits, q_off, out_off, n_el)
    form = U.ukv_get_param(db.pool, U.UKV_PARAM_PREFILL_FORM_USED)
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    U.ukv_profile_read(db.pool)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    prof = U.ukv_profile_read(db.pool)
    k_ms = prof.prefill_ms / max(prof.n_prefill, 1)
    # causal attention: row p of a prompt meets p + 1 tokens; 2 products x 2 flop x d per (row, token, query head)
    flops = float(sum(4.0 * s.head_dim * s.n_q_heads * (int(c) * (int(c) + 1) / 2)
                      for s, c in ((b.service_of(i), b.ctx_len[i]) for i in range(b.n_requests))))
    tokens = int(ctx.sum())
    line = {
        "metric": "prefill-attention TFLOP/s (causal, paged KV), 1 GPU", "value": round(flops * args.steps / wall / 1e12, 2),
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if form == 2 else "bf16 scores, fp16 weights x fp16 V", "data": "synthetic",
        "config": {"workload": f"prefill/{args.prefill_workload}: {n} whole prompts, services {names}, lengths {law}",
                   "prompt_tokens": tokens, "flops_per_step": flops, "page_bytes": b.page_bytes,
                   "softmax_weights": "two bf16 parts" if form == 2 else "one fp16 part (step includes the fp16 copy of V)"},
        "prompt_tokens_per_s": round(tokens * args.steps / wall, 1),
        "kernel_ms": {"prefill": round(k_ms, 4)},
        "roofline": {"bound": "mfma", "kernel": "prefill_kernel", "achieved": round(flops / (k_ms * 1e-3) / 1e12, 2),
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(flops / (k_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None},
    }
    db.close()
    print(json.dumps(line))


def main_grid(args):
    """Decode attention on uniform batches: n requests of one service, all of the same context length, from one
    short request to a full device.  Shows where the launch is latency-bound (few, short requests), how a single
    long request is spread over the device by the split-KV plan, and the rate the kernel reaches when the batch
    is large and even.  One JSON line: cells of (service, requests, tokens) -> microseconds of decode + merge
    kernels (HIP events on the dispatches) and KV TB/s."""
    import numpy as np
    import torch
    import paper_2504_15720_amd as U
    from synth import SHAPES
    from synth.workloads import normal_bf16

    dev = torch.device("cuda:0")
    PAGE = 16384
    noise = torch.from_numpy(normal_bf16(1 << 22, np.random.default_rng(1)).view(np.int16)).to(dev)
    stream = torch.cuda.current_stream().cuda_stream
    cells = []
    for name in ("7b", "70b", "h12"):
        sv = SHAPES[name]
        row = sv.n_q_heads * sv.head_dim
        for n in (1, 2, 4, 8, 16, 64):
            for ctx in (1024, 4096, 16384, 65536):
                n_pg = -(-ctx * sv.token_bytes // PAGE)
                n_pages = n * n_pg + 64
                if n_pages * PAGE > 40e9:
                    continue
                raw = torch.empty(n_pages * PAGE // 2 + PAGE // 2, dtype=torch.int16, device=dev)
                skip = (-raw.data_ptr() % PAGE) // 2
                pool_t = raw[skip:skip + n_pages * PAGE // 2]
                pool_t.copy_(noise.repeat(-(-pool_t.numel() // noise.numel()))[:pool_t.numel()])
                table_t = torch.from_numpy(np.random.default_rng(2).permutation(n_pages)[:n * n_pg].astype(np.int32)).to(dev)
                pool = U.ukv_pool_create(pool_t.data_ptr(), n_pages * PAGE, PAGE, [sv])
                U.ukv_set_param(pool, U.UKV_PARAM_PROFILE, 1)
                q_t = noise[:n * row].clone()
                out_t = torch.zeros(n * row, dtype=torch.float32, device=dev)
                ws = U.ukv_decode_workspace_bytes(pool, n)
                ws_t = torch.empty(ws, dtype=torch.uint8, device=dev)
                off = (np.arange(n) * row).astype(np.uint64)
                desc = U.BatchDesc([0] * n, [ctx] * n, (np.arange(n) * n_pg).astype(np.uint64), table_t.data_ptr(),
                                   q_t.data_ptr(), off, out_t.data_ptr(), off)
                for _ in range(3):
                    U.ukv_decode_attention(pool, desc, ws_t.data_ptr(), ws, stream)
                torch.cuda.synchronize()
                U.ukv_profile_read(pool)
                for _ in range(args.steps):
                    U.ukv_decode_attention(pool, desc, ws_t.data_ptr(), ws, stream)
                torch.cuda.synchronize()
                pr = U.ukv_profile_read(pool)
                us = 1e3 * (pr.decode_ms / pr.n_decode + (pr.reduce_ms / pr.n_reduce if pr.n_reduce else 0.0))
                kv = n * ctx * sv.token_bytes
                cells.append({"service": f"{sv.n_q_heads}/{sv.n_kv_heads} d={sv.head_dim}", "requests": n, "tokens": ctx,
                              "kv_mb": round(kv / 1e6, 1), "kernels_us": round(us, 1), "tb_s": round(kv / us / 1e6, 2)})
                torch.cuda.synchronize()
                U.ukv_pool_destroy(pool)
                del raw, pool_t
    print(json.dumps({"metric": "decode attention on uniform batches: decode + merge kernel time, 1 GPU", "unit": "us",
                      "steps": args.steps, "data": "synthetic", "page_bytes": PAGE, "cells": cells}))

    # the same for prefill attention: n whole prompts of one length
    cells = []
    for name in ("7b", "70b", "h12"):
        sv = SHAPES[name]
        row = sv.n_q_heads * sv.head_dim
        for n in (1, 4, 16):
            for ctx in (512, 2048, 8192, 32768):
                if n * ctx * row * 6 > 30e9:
                    continue
                n_pg = -(-ctx * sv.token_bytes // PAGE)
                n_pages = n * n_pg + 64
                raw = torch.empty(n_pages * PAGE // 2 + PAGE // 2, dtype=torch.int16, device=dev)
                skip = (-raw.data_ptr() % PAGE) // 2
                pool_t = raw[skip:skip + n_pages * PAGE // 2]
                pool_t.copy_(noise.repeat(-(-pool_t.numel() // noise.numel()))[:pool_t.numel()])
                table_t = torch.from_numpy(np.random.default_rng(2).permutation(n_pages)[:n * n_pg].astype(np.int32)).to(dev)
                pool = U.ukv_pool_create(pool_t.data_ptr(), n_pages * PAGE, PAGE, [sv])
                U.ukv_set_param(pool, U.UKV_PARAM_PROFILE, 1)
                q_t = noise.repeat(-(-n * ctx * row // noise.numel()))[:n * ctx * row].contiguous()
                out_t = torch.empty(n * ctx * row, dtype=torch.float32, device=dev)
                ws = U.ukv_prefill_workspace_bytes_one_part(pool, n, n * ctx, n * ctx)   # room for either form of the weights
                ws_t = torch.empty(ws, dtype=torch.uint8, device=dev)
                off = (np.arange(n) * ctx * row).astype(np.uint64)
                desc = U.BatchDesc([0] * n, [ctx] * n, (np.arange(n) * n_pg).astype(np.uint64), table_t.data_ptr(),
                                   q_t.data_ptr(), off, out_t.data_ptr(), off)
                q_len = np.full(n, ctx, np.uint32)
                for _ in range(2):
                    U.ukv_prefill_attention(pool, desc, q_len, ws_t.data_ptr(), ws, stream)
                torch.cuda.synchronize()
                U.ukv_profile_read(pool)
                n_calls = max(5, args.steps)
                t0 = time.perf_counter()
                for _ in range(n_calls):
                    U.ukv_prefill_attention(pool, desc, q_len, ws_t.data_ptr(), ws, stream)
                torch.cuda.synchronize()
                call_us = (time.perf_counter() - t0) / n_calls * 1e6    # whole call: upload, fp16 copy of V if any, kernel
                pr = U.ukv_profile_read(pool)
                us = 1e3 * pr.prefill_ms / pr.n_prefill
                flops = n * 4.0 * row * ctx * (ctx + 1) / 2            # causal, counted once
                cells.append({"service": f"{sv.n_q_heads}/{sv.n_kv_heads} d={sv.head_dim}", "prompts": n, "tokens": ctx,
                              "weights_parts": U.ukv_get_param(pool, U.UKV_PARAM_PREFILL_FORM_USED),
                              "kernel_us": round(us, 1), "call_us": round(call_us, 1), "tflops": round(flops / us / 1e6, 1)})
                torch.cuda.synchronize()
                U.ukv_pool_destroy(pool)
                del raw, pool_t, q_t, out_t
    print(json.dumps({"metric": "prefill attention on uniform batches of whole prompts: prefill kernel time, 1 GPU",
                      "unit": "us", "steps": max(5, args.steps), "data": "synthetic", "page_bytes": PAGE, "cells": cells}))

    # Chunks of long prompts: q_len rows of n requests against 16384 cached tokens (the chunk's own included), where
    # few workgroups would each walk the whole context; with the room for partial results in the workspace
    # ("stretches") and without it (one workgroup per tile of rows).
    cells = []
    ctx = 16384
    for name in ("7b", "70b"):
        sv = SHAPES[name]
        row = sv.n_q_heads * sv.head_dim
        for n, ql in ((1, 128), (1, 512), (1, 2048), (8, 512)):
            n_pg = -(-ctx * sv.token_bytes // PAGE)
            n_pages = n * n_pg + 64
            raw = torch.empty(n_pages * PAGE // 2 + PAGE // 2, dtype=torch.int16, device=dev)
            skip = (-raw.data_ptr() % PAGE) // 2
            pool_t = raw[skip:skip + n_pages * PAGE // 2]
            pool_t.copy_(noise.repeat(-(-pool_t.numel() // noise.numel()))[:pool_t.numel()])
            table_t = torch.from_numpy(np.random.default_rng(2).permutation(n_pages)[:n * n_pg].astype(np.int32)).to(dev)
            pool = U.ukv_pool_create(pool_t.data_ptr(), n_pages * PAGE, PAGE, [sv])
            U.ukv_set_param(pool, U.UKV_PARAM_PROFILE, 1)
            q_t = noise.repeat(-(-n * ql * row // noise.numel()))[:n * ql * row].contiguous()
            out_t = torch.empty(n * ql * row, dtype=torch.float32, device=dev)
            ws_small = U.ukv_prefill_workspace_bytes(pool, n, n * ql)
            ws_full = U.ukv_prefill_workspace_bytes_one_part(pool, n, n * ql, n * ctx)
            ws_t = torch.empty(ws_full, dtype=torch.uint8, device=dev)
            off = (np.arange(n) * ql * row).astype(np.uint64)
            desc = U.BatchDesc([0] * n, [ctx] * n, (np.arange(n) * n_pg).astype(np.uint64), table_t.data_ptr(),
                               q_t.data_ptr(), off, out_t.data_ptr(), off)
            q_len = np.full(n, ql, np.uint32)
            cell = {"service": f"{sv.n_q_heads}/{sv.n_kv_heads} d={sv.head_dim}", "requests": n, "cached_tokens": ctx, "q_len": ql}
            for label, ws in (("stretches", ws_full), ("one_workgroup_per_tile", ws_small)):
                for _ in range(2):
                    U.ukv_prefill_attention(pool, desc, q_len, ws_t.data_ptr(), ws, stream)
                torch.cuda.synchronize()
                U.ukv_profile_read(pool)
                n_calls = max(30, args.steps)
                t0 = time.perf_counter()
                for _ in range(n_calls):
                    U.ukv_prefill_attention(pool, desc, q_len, ws_t.data_ptr(), ws, stream)
                torch.cuda.synchronize()
                call_us = (time.perf_counter() - t0) / n_calls * 1e6
                pr = U.ukv_profile_read(pool)
                cell[label] = {"kernel_us": round(1e3 * pr.prefill_ms / pr.n_prefill, 1), "call_us": round(call_us, 1),
                               "partials": U.ukv_get_param(pool, U.UKV_PARAM_PREFILL_PARTIALS_USED),
                               "weights_parts": U.ukv_get_param(pool, U.UKV_PARAM_PREFILL_FORM_USED)}
            cells.append(cell)
            U.ukv_pool_destroy(pool)
            del raw, pool_t, q_t, out_t, ws_t
    print(json.dumps({"metric": "prefill attention on chunks of long prompts: prefill kernel and whole-call time, 1 GPU",
                      "unit": "us", "steps": max(5, args.steps), "data": "synthetic", "page_bytes": PAGE, "cells": cells}))


def main_serve(args):
    """Serving loop over the unified cache driven by the doubling-budget scheduler (section 4.2): requests of
    three services arrive at once, are prefilled (bulk store + prefill attention) and decoded to their output
    lengths; pages come from the pool's free list and go back when a request finishes.  Policies and clocks:
    see paper_2504_15720_amd/serving.py.  Prints one JSON line per policy.  One attention layer; no model around it."""
    from paper_2504_15720_amd.serving import ServingLoop
    from synth.serving import draw_serve_workload, modelled_time

    wl = draw_serve_workload(args.serve_requests)
    loop = ServingLoop(wl, modelled_time)
    loop.run("mixed", clock=args.serve_clock)                   # warm-up: first launches, staging buffers
    for policy in ("db", "mixed"):
        r = loop.run(policy, clock=args.serve_clock)
        print(json.dumps({
            "metric": "serving loop, generated tokens/s (one attention layer), 1 GPU",
            "value": round(r["generated_tokens"] / r["wall_s"], 1), "unit": "tokens/s", "n_gpus": 1,
            "higher_is_better": True, "data": "synthetic", "dtype": "f32",
            "config": {"workload": f"serve: 3 services (32/32, 40/40, 32/8 heads, d=128) x {args.serve_requests} requests "
                                   f"at t=0, prompts lognormal 256/1024/512, outputs lognormal 32/96/64",
                       "policy": policy, "clock": args.serve_clock, "max_batch": wl.max_batch, "pool_pages": wl.n_pages},
            "wall_s": round(r["wall_s"], 4), "iterations": r["iterations"], "launch_groups": r["launch_groups"],
            "generated_tokens": r["generated_tokens"], "prompt_tokens": r["prompt_tokens"],
            "mean_latency_per_output_token_ms": r["mean_latency_per_output_token_ms"]}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, help="workload 1..5 (default: the two-service batch)")
    ap.add_argument("--block", type=int, default=0, help="decode workgroup size override (256/512)")
    ap.add_argument("--max-spans", type=int, default=0)
    ap.add_argument("--min-span-bytes", type=int, default=0)
    ap.add_argument("--heads-per-slice", type=int, default=0)
    ap.add_argument("--slots", type=int, default=0)
    ap.add_argument("--no-taper", action="store_true")
    ap.add_argument("--separate-append", action="store_true")
    ap.add_argument("--replan-each-step", action="store_true",
                    help="ukv_decode_step in every step (host plan + upload) instead of the plan kept across steps")
    ap.add_argument("--replan-every", type=int, default=-1, help="UKV_PARAM_REPLAN_EVERY")
    ap.add_argument("--merge-acq-rel", action="store_true", help="UKV_PARAM_MERGE_ACQ_REL = 1")
    ap.add_argument("--validate", action="store_true", help="UKV_PARAM_VALIDATE = 1 (page tables checked before every call)")
    ap.add_argument("--phase", choices=["decode", "prefill", "serve", "grid"], default="decode")
    ap.add_argument("--serve-requests", type=int, default=64, help="requests per service of the serving loop")
    ap.add_argument("--serve-clock", choices=["wall", "model"], default="wall",
                    help="time charged to the scheduler's budgets: measured wall time, or a model of the batch (reproducible)")
    ap.add_argument("--prefill-workload", choices=list(PREFILL_WORKLOADS), default="chat")
    ap.add_argument("--prefill-no-xcd", action="store_true")
    ap.add_argument("--prefill-weights", type=int, choices=[0, 1, 2], default=0,
                    help="form of the softmax weights: 0 = the library's choice, 1 = one fp16 part, 2 = two bf16 parts")
    ap.add_argument("--taper", type=int, default=0)
    ap.add_argument("--gqa-cost-pct", type=int, default=0)
    ap.add_argument("--unfused-merge", action="store_true", help="merge split partials in a second launch")
    ap.add_argument("--fused-merge", action="store_true",
                    help="merge split partials inside the decode launch also where the pool's default is the second launch")
    ap.add_argument("--layout", choices=["merged", "split"], default="merged",
                    help="split = one block stream and table per (request, kv head), the alternative of section 4.4")
    ap.add_argument("--split-page-bytes", type=int, default=0, help="block size of the split layout")
    ap.add_argument("--as-stated-pool", action="store_true",
                    help="keep the pool at the workload's stated size and admit requests in draw order while pages remain")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--attention-only", action="store_true", help="skip grow+append in the step (diagnostic)")
    ap.add_argument("--time-every", type=int, default=4,
                    help="decode phase: HIP-event timing of every n-th launch of each kernel (a timed launch costs "
                         "about 10 us of stream time; 1 = every launch)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; every GPU box here has one and the path uses no "
              "collectives. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    if args.steps < 3 * args.time_every:      # short runs (profiler passes): time every launch
        args.time_every = 1
    if args.phase == "prefill":
        return main_prefill(args)
    if args.phase == "serve":
        return main_serve(args)
    if args.phase == "grid":
        return main_grid(args)

    import numpy as np
    import torch
    import paper_2504_15720_amd as U
    from synth import make_config
    from paper_2504_15720_amd.device_batch import DeviceBatch

    assert torch.cuda.is_available(), "bench.py needs a GPU (there is no CPU path)"
    t_gen = time.perf_counter()
    # tables must have room for every step's new token
    b = make_config(args.config, reserve_tokens=args.steps + args.warmup + 1, fill_pool=args.layout == "merged",
                    as_stated=args.as_stated_pool)
    if args.layout == "split":
        from synth import to_split_layout
        b = to_split_layout(b, pool_seed=7, page_bytes=args.split_page_bytes or None)
    t_gen = time.perf_counter() - t_gen
    db = DeviceBatch(b, profile=args.time_every)
    if args.block:
        U.ukv_set_param(db.pool, U.UKV_PARAM_BLOCK_THREADS, args.block)
    if args.max_spans:
        U.ukv_set_param(db.pool, U.UKV_PARAM_MAX_SPANS, args.max_spans)
    if args.min_span_bytes:
        U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, args.min_span_bytes)
    if args.heads_per_slice:
        U.ukv_set_param(db.pool, U.UKV_PARAM_HEADS_PER_SLICE, args.heads_per_slice)
    if args.slots:
        U.ukv_set_param(db.pool, U.UKV_PARAM_SLOTS, args.slots)
    if args.taper:
        U.ukv_set_param(db.pool, U.UKV_PARAM_TAPER, args.taper)
    if args.gqa_cost_pct:
        U.ukv_set_param(db.pool, U.UKV_PARAM_GQA_COST_PCT, args.gqa_cost_pct)
    if args.no_taper:
        U.ukv_set_param(db.pool, U.UKV_PARAM_TAPER, 0)
    if args.unfused_merge:
        U.ukv_set_param(db.pool, U.UKV_PARAM_FUSED_MERGE, 0)
    if args.fused_merge:
        U.ukv_set_param(db.pool, U.UKV_PARAM_FUSED_MERGE, 1)
    if args.validate:
        U.ukv_set_param(db.pool, U.UKV_PARAM_VALIDATE, 1)
    if args.merge_acq_rel:
        U.ukv_set_param(db.pool, U.UKV_PARAM_MERGE_ACQ_REL, 1)
    if args.replan_every >= 0:
        U.ukv_set_param(db.pool, U.UKV_PARAM_REPLAN_EVERY, args.replan_every)
    db.resize_workspace()
    rng = np.random.default_rng(1)
    _, nk, nv = b.draw_step_inputs(rng)
    db.set_new(nk, nv)
    kept_plan = not (args.attention_only or args.separate_append or args.replan_each_step)
    if kept_plan:
        db.make_plan()

    kv_bytes = []

    def step():
        if args.attention_only:
            desc = db.desc()
        else:
            entry, ids = b.grow_one_token()
            if ids.size:
                lib_ids = U.ukv_pages_alloc(db.pool, ids.size)
                assert np.array_equal(lib_ids, ids)
            if kept_plan:
                db.plan_step(ids)
                kv_bytes.append(b.kv_bytes())
                return
            desc = db.desc(entry, ids)
            if args.separate_append:
                db.append(desc)
            else:
                db.step(desc)
                kv_bytes.append(b.kv_bytes())
                return
        db.decode(desc)
        kv_bytes.append(b.kv_bytes())

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    U.ukv_profile_read(db.pool)          # drop warm-up kernel times
    kv_bytes.clear()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    prof = U.ukv_profile_read(db.pool)

    total_kv = float(sum(kv_bytes))
    kv_per_step = total_kv / args.steps
    value = total_kv / wall / 1e9
    dec_ms = prof.decode_ms / max(prof.n_decode, 1)
    red_ms = prof.reduce_ms / max(prof.n_reduce, 1) if prof.n_reduce else 0.0
    app_ms = prof.append_ms / max(prof.n_append, 1) if prof.n_append else 0.0
    achieved = kv_per_step / (dec_ms * 1e-3) / 1e9
    info, _ = U.ukv_plan_decode(db.pool, db.desc(), want_items=False)

    line = {
        "metric": "decode-attention KV GB/s, mixed-service batch, 1 GPU",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": WORKLOAD_NAMES[args.config] + (", pool as stated: requests admitted in draw order while pages remain"
                                                              if args.as_stated_pool else ""),
                   "n_requests": b.n_requests, "drawn_requests": b.notes.get("drawn_requests", b.n_requests),
                   "kv_bytes_per_step": int(kv_per_step), "pool_pages": b.n_pages,
                   "stated_pool_pages": b.notes.get("stated_pages"), "page_bytes": b.page_bytes,
                   "step": "attention only" if args.attention_only else
                           "grow + append + attention (two calls)" if args.separate_append else
                           ("grow + append + attention, plan kept across steps (one launch)" if kept_plan else
                            "grow + append + attention, planned and uploaded every step (upload + one launch)") +
                           ("" if U.ukv_get_param(db.pool, U.UKV_PARAM_FUSED_MERGE) else
                            " + merge of split partials (second launch)"),
                   "layout": args.layout, "block_table_entries": int(b.pages_owned().sum()),
                   "pages_in_use": int(b.stack.used_pages),
                   "internal_waste_bytes": int(b.pages_owned().sum()) * int(b.page_bytes) - int(b.kv_bytes()),
                   "kv_storage": "bf16", "decode_workgroups": info.n_spans, "work_items": info.n_items,
                   "block_threads": U.ukv_get_param(db.pool, U.UKV_PARAM_BLOCK_THREADS)},
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "tokens_per_s": round(b.n_requests * args.steps / wall, 1),
        "kernel_ms": {"decode": round(dec_ms, 4), "reduce": round(red_ms, 4), "append": round(app_ms, 4)},
        "kernel_ms_launches_timed": {"decode": prof.n_decode, "every": args.time_every},
        "attention_kernels_gbs": round(kv_per_step / ((dec_ms + red_ms) * 1e-3) / 1e9, 2),
        "roofline": {"bound": "hbm", "kernel": "decode_kernel", "achieved": round(achieved, 2),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": read_traffic(args.config)[0] if not args.as_stated_pool and args.layout == "merged" else None,
                     "traffic_source": read_traffic(args.config)[1]},
        "setup_s": round(t_gen, 1),
    }
    if kv_per_step < 256e6:  # smaller than the 256 MB of last-level cache: the launch never goes to HBM
        line["note"] = "working set is cache resident: the GB/s here is not an HBM figure (launch-bound workload)"
        line["roofline"]["note"] = "cache resident, not HBM"
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(b, int(kv_per_step), one_thread=args.config in (1, 2))
        line["cpu_baseline"]["value"] = round(line["cpu_baseline"]["value"], 4)
        line["cpu_baseline"]["tokens_per_s"] = round(line["cpu_baseline"]["tokens_per_s"], 2)
    db.close()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
