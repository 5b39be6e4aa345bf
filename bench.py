#!/usr/bin/env python3
"""Benchmark of the fused Adam(W) bucket step on one MI355X.

A "step" is one pass of the whole optimizer hot path over the Llama-3-8B-shaped state
(8,030,261,248 parameters in 81 flat buckets of 100 M elements, everything resident in HBM):
stage-1 gradient statistics over all buckets, stage-2 reduction with the GPU-side validation
outcome (norm, NaN/Inf flag, clip coefficient), and the fused AdamW + bf16-cast step over all
buckets in one launch, clipped at max_norm = 1.0 -- with no host round trip in between.
Gradients are regenerated from the seed before every step, outside the timed region (they
stand in for the backward pass).  Each timed step is bracketed by torch.cuda.synchronize().

Prints ONE JSON line: metric "adam_step_params_per_s" with a roofline object for the
dominant kernel (the fused step, 28 algorithmic bytes per parameter) and a cpu_baseline
object (the scalar CPU oracle timed on a bounded sample of the same workload).
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

HBM_PEAK_GBPS = 8000.0
STEP_BYTES_PER_PARAM = 28          # read g 2 + p,m,v 12 ; write p,m,v 12 + bf16 copy 2
STATS_BYTES_PER_PARAM = 2


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic(name):
    """HBM bytes per launch of the step kernel from the committed rocprofv3 counter summary
    (profiles/<name>), if present: a line 'traffic_bytes_per_launch = <number>'."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1].split()[0])
    except OSError:
        pass
    return None


def cpu_baseline(cfg, total, bucket, seed_step, threads, sample):
    """Time the CPU oracle (validation + step, one iteration) on the first `sample` parameters
    of the workload, split statically over `threads` host threads."""
    import numpy as np
    import torch
    import oracle
    import synth
    chunk = 1 << 24
    obs, grads, start = [], [], 0
    while start < sample:
        n = min(chunk, sample - start)
        p = synth.normal_f32(cfg["seed"], synth.STREAM_PARAM, 0, start, n, cfg["sigma_p"], "cuda")
        g = synth.normal_16bit(cfg["seed"], synth.STREAM_GRAD, seed_step, start, n, cfg["sigma_g"],
                               torch.bfloat16, "cuda")
        obs.append(oracle.Bucket(p.cpu().numpy()))
        grads.append(g.cpu().view(torch.int16).numpy().view(np.uint16).copy())
        start += n
    tr = oracle.Trainer(obs, max_norm=cfg["max_norm"], threads=threads, **cfg["hp"])
    t0 = time.perf_counter()
    tr.iteration(grads)
    dt = time.perf_counter() - t0
    return {"value": sample / dt, "unit": "params/s", "cores": threads, "kind": "oracle",
            "sample": f"first {sample} parameters of the workload, one iteration "
                      f"(global norm + NaN/Inf check + clipped AdamW step), {dt:.2f} s wall"}


def stream_bench(args):
    """Workload 4: fp32 p, m, v in pinned host memory, streamed through device staging slots
    with so_stream_step; gradients and the bf16 working copy stay on the GPU.  The full
    workload needs 280 GB of pinned host memory; --layers cuts the 48 layers down to what the
    machine can pin (the deviation is reported in the JSON line)."""
    import torch
    import synth
    from paper_2509_21271_amd import binding as B

    torch.cuda.set_device(0)
    cfg = synth.config(4)
    total = synth.total_params(4, args.layers)
    bucket = cfg["bucket"]
    hp = B.hparams(cfg["hp"]["lr"], cfg["hp"]["beta1"], cfg["hp"]["beta2"], cfg["hp"]["eps"], cfg["hp"]["wd"])
    log(f"workload {cfg['name']} with {args.layers} of 48 layers: {total} params, "
        f"{12 * total / 1e9:.1f} GB of {'pageable' if args.unpinned else 'pinned'} host state")
    if args.unpinned:     # pageable host memory: what Sec. 4.5 warns against, for comparison
        pinned = []
        host = [torch.empty(total, dtype=torch.float32) for _ in range(3)]
    else:
        pinned = [B.PinnedArray(total) for _ in range(3)]     # exact size: torch's pinned pool rounds up
        host = [a.t for a in pinned]
    host[1].zero_()
    host[2].zero_()
    g = torch.empty(total, dtype=torch.bfloat16, device="cuda")
    q = torch.zeros(total, dtype=torch.bfloat16, device="cuda")
    ranges = [(s, min(bucket, total - s)) for s in range(0, total, bucket)]
    for s, n in ranges:
        host[0][s:s + n].copy_(synth.normal_f32(cfg["seed"], synth.STREAM_PARAM, 0, s, n, cfg["sigma_p"], "cuda"))
    ctx = B.so_create(0, torch.cuda.current_stream().cuda_stream)
    st = B.so_stream_state()
    st.host_param, st.host_exp_avg, st.host_exp_avg_sq = (h.data_ptr() for h in host)
    st.grad, st.param_lp = g.data_ptr(), q.data_ptr()
    st.n_total, st.bucket_elems, st.grad_dtype = total, bucket, B.SO_GRAD_BF16
    # --resident-buckets N: N more buckets keep their state on the GPU and are stepped in the
    # shadow of the transfers (the repartitioned step of Sec. 4.3).
    resident, keep = [], []
    for j in range(args.resident_buckets):
        off = total + j * bucket
        rp = synth.normal_f32(cfg["seed"], synth.STREAM_PARAM, 0, off, bucket, cfg["sigma_p"], "cuda")
        rg = synth.normal_16bit(cfg["seed"], synth.STREAM_GRAD, 1, off, bucket, cfg["sigma_g"], torch.bfloat16, "cuda")
        rm, rv = torch.zeros_like(rp), torch.zeros_like(rp)
        rq = torch.zeros(bucket, dtype=torch.bfloat16, device="cuda")
        keep.append((rp, rg, rm, rv, rq))
        resident.append(B.bucket_of(rg, rp, rm, rv, rq))
    n_res = args.resident_buckets * bucket
    reps = []
    t_adam = 1
    for k in range(args.warmup + args.steps):
        for s, n in ranges:
            g[s:s + n] = synth.normal_16bit(cfg["seed"], synth.STREAM_GRAD, t_adam, s, n, cfg["sigma_g"],
                                            torch.bfloat16, "cuda")
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if resident:
            rep, res_ms = B.so_hybrid_step(ctx, st, resident, hp, t_adam, 1.0)
        else:
            rep, res_ms = B.so_stream_step(ctx, st, hp, t_adam, 1.0), 0.0
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        log(f"step {t_adam}: {1e3 * dt:.0f} ms  H2D {rep.h2d_gbps:.1f}  D2H {rep.d2h_gbps:.1f} GB/s  "
            f"kernels {rep.kernel_ms:.1f} ms  resident part {res_ms:.1f} ms")
        if k >= args.warmup:
            reps.append((dt, rep.h2d_gbps, rep.d2h_gbps, rep.kernel_ms, res_ms))
        t_adam += 1
    separate = None
    if resident:        # the same two parts one after the other, for comparison
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        B.so_stream_step(ctx, st, hp, t_adam, 1.0)
        t1 = time.perf_counter()
        B.so_adam_step_multi(ctx, resident, hp, t_adam, 1.0)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        separate = {"stream_ms": 1e3 * (t1 - t0), "resident_ms": 1e3 * (t2 - t1)}
        log(f"separately: streamed {separate['stream_ms']:.0f} ms + resident {separate['resident_ms']:.1f} ms")
    B.so_destroy(ctx)
    host = None
    for a in pinned:
        a.free()
    ms = 1e3 * sum(r[0] for r in reps) / len(reps)
    out = {"metric": "adam_stream_step_params_per_s", "value": (total + n_res) / (ms * 1e-3), "unit": "params/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
           "data": "synthetic",
           "config": {"workload": f"{cfg['name']} ({args.layers} of 48 layers)", "params": total,
                      "bucket_elems": bucket, "buckets": len(ranges), "host_state_gb": 12 * total / 1e9,
                      "host_memory": "pageable" if args.unpinned else "pinned",
                      "deviation": "layer count reduced to fit the machine's pinned-memory limit"
                      if args.layers < 48 else None},
           "h2d_gbps": sum(r[1] for r in reps) / len(reps), "d2h_gbps": sum(r[2] for r in reps) / len(reps),
           "link_gbps_both_directions": 24 * total / (ms * 1e-3) / 1e9,
           "step_kernels_ms": sum(r[3] for r in reps) / len(reps)}
    if resident:
        out["config"]["resident_buckets"] = args.resident_buckets
        out["config"]["resident_params"] = n_res
        out["resident_part_ms"] = sum(r[4] for r in reps) / len(reps)
        out["separate_calls"] = separate
    print(json.dumps(out), flush=True)


def repartition_plan(args):
    """The bucket-repartitioning inequality of Sec. 4.3 on this machine's measured times: how
    many of the last buckets must keep their optimizer state on the GPU so that the offloaded
    path of one bucket (move in, step, move out) hides behind the backward pass and resident
    step of those buckets.  The three offloaded-path times and the resident step time of one
    200 M-element bucket are measured; the backward time per bucket depends on model and batch,
    so a range is tabulated."""
    import torch
    import synth
    from paper_2509_21271_amd import binding as B

    torch.cuda.set_device(0)
    cfg = synth.config(4)
    bucket = cfg["bucket"]
    hp = B.hparams(cfg["hp"]["lr"], cfg["hp"]["beta1"], cfg["hp"]["beta2"], cfg["hp"]["eps"], cfg["hp"]["wd"])
    pinned = [B.PinnedArray(bucket) for _ in range(3)]
    for a in pinned:
        a.t.zero_()
    dev = [torch.zeros(bucket, dtype=torch.float32, device="cuda") for _ in range(3)]
    g = synth.normal_16bit(cfg["seed"], synth.STREAM_GRAD, 1, 0, bucket, cfg["sigma_g"], torch.bfloat16, "cuda")
    q = torch.zeros(bucket, dtype=torch.bfloat16, device="cuda")
    ctx = B.so_create(0, torch.cuda.current_stream().cuda_stream)

    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t0) / reps

    move_in = timed(lambda: [d.copy_(a.t, non_blocking=True) for d, a in zip(dev, pinned)])
    move_out = timed(lambda: [a.t.copy_(d, non_blocking=True) for d, a in zip(dev, pinned)])
    bk = B.bucket_of(g, dev[0], dev[1], dev[2], q)
    t = [1]

    def step():
        B.so_adam_step(ctx, bk, hp, t[0], 1.0)
        t[0] += 1

    step_ms = timed(step, 20)
    B.so_destroy(ctx)
    for a in pinned:
        a.free()
    n_buckets = -(-synth.total_params(4) // bucket)
    rows = []
    for bwd in (1.0, 2.0, 5.0, 10.0, 20.0, 50.0):
        n = B.so_plan_resident(move_in, step_ms, move_out, bwd, step_ms, n_buckets, n_buckets)
        rows.append({"bwd_ms_per_bucket": bwd, "n_resident": n})
        log(f"backward {bwd:5.1f} ms per bucket -> keep the last {n} of {n_buckets} buckets on the GPU")
    print(json.dumps({"metric": "resident_buckets_from_the_repartitioning_inequality", "unit": "buckets",
                      "n_gpus": 1, "data": "synthetic", "dtype": "f32", "vs_baseline": None,
                      "config": {"workload": f"{cfg['name']}: one bucket of {bucket} parameters measured, "
                                             f"{n_buckets} buckets in all"},
                      "measured_ms": {"move_in_12B_per_param": move_in, "step": step_ms,
                                      "move_out_12B_per_param": move_out},
                      "rows": rows}), flush=True)


def bucket_sweep(args):
    """Host-link rate of the streamed step as a function of the staged bucket size (the
    paper's bandwidth-versus-tensor-size study, Sec. 4.3, on this machine's host link):
    2^30 parameters of pinned state, bucket sizes from 256 Ki to 256 Mi elements."""
    import torch
    from paper_2509_21271_amd import binding as B

    torch.cuda.set_device(0)
    total = 1 << 30
    pinned = [B.PinnedArray(total) for _ in range(3)]
    for a in pinned:
        a.t.zero_()
    g = torch.zeros(total, dtype=torch.bfloat16, device="cuda")
    q = torch.zeros(total, dtype=torch.bfloat16, device="cuda")
    ctx = B.so_create(0, torch.cuda.current_stream().cuda_stream)
    hp = B.hparams(1e-4, 0.9, 0.999, 1e-8, 0.01)
    st = B.so_stream_state()
    st.host_param, st.host_exp_avg, st.host_exp_avg_sq = (a.ptr for a in pinned)
    st.grad, st.param_lp = g.data_ptr(), q.data_ptr()
    st.n_total, st.grad_dtype = total, B.SO_GRAD_BF16
    rows = []
    for lg in range(28, 17, -1):            # largest first: the staging slots are allocated once
        st.bucket_elems = 1 << lg
        B.so_stream_step(ctx, st, hp, 1, 1.0)
        best = None
        for rep in range(2):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            r = B.so_stream_step(ctx, st, hp, 2 + rep, 1.0)
            dt = time.perf_counter() - t0
            if best is None or dt < best[0]:
                best = (dt, r.h2d_gbps, r.d2h_gbps)
        rows.append({"bucket_elems": 1 << lg, "bucket_mb_fp32": (4 << lg) / 1e6, "ms": 1e3 * best[0],
                     "h2d_gbps": best[1], "d2h_gbps": best[2], "link_gbps": 24 * total / best[0] / 1e9})
        log(f"bucket 2^{lg} elements ({(4 << lg) / 1e6:8.1f} MB per fp32 array): {1e3 * best[0]:8.1f} ms  "
            f"H2D {best[1]:5.1f}  D2H {best[2]:5.1f}  both {24 * total / best[0] / 1e9:5.1f} GB/s")
    B.so_destroy(ctx)
    for a in pinned:
        a.free()
    print(json.dumps({"metric": "stream_step_link_gbps_vs_bucket_size", "unit": "GB/s", "n_gpus": 1,
                      "data": "synthetic", "config": {"workload": "2^30 parameters, pinned host state"},
                      "rows": rows}), flush=True)


def cast_variants(args):
    """The casting question of Sec. 4.5 on this machine's host link: fp32 master parameters in
    host memory, 16-bit working copy wanted on the GPU.
      cast on the GPU   move fp32 (4 B/param) in chunks through staging slots, cast each chunk
                        there while the next is on its way: so_stream_cast_params, all of it
                        this library's code
      cast on the host  cast to bf16 on the host cores, then move 2 B/param.  The host cast is
                        NOT this library's (it has no CPU path): torch's own conversion on the
                        job's host threads stands in for it, into a pinned buffer (best case) and
                        into a fresh pageable tensor (what a framework's `.to(bf16).cuda()` does)
    for tensor sizes from 1 MB to 2 GB of fp32."""
    import torch
    from paper_2509_21271_amd import binding as B

    torch.cuda.set_device(0)
    threads = min(16, os.cpu_count() or 1)
    torch.set_num_threads(threads)
    nmax = 1 << 29
    src = B.PinnedArray(nmax)
    src.t.normal_(0.0, 0.02)
    half_store = B.PinnedArray(nmax // 2)                       # 2 * nmax bytes of pinned memory
    half = half_store.t.view(torch.bfloat16)
    q = torch.zeros(nmax, dtype=torch.bfloat16, device="cuda")
    ctx = B.so_create(0, torch.cuda.current_stream().cuda_stream)
    B.so_stream_cast_params(ctx, src.ptr, q.data_ptr(), nmax, 1 << 24)      # staging slots allocated here

    def best_of(fn, reps):
        return min(fn() for _ in range(reps))

    rows = []
    for lg in range(18, 30):
        n = 1 << lg
        reps = 5 if lg < 26 else 3
        chunk = min(n, 1 << 24)
        gpu_ms = best_of(lambda: B.so_stream_cast_params(ctx, src.ptr, q.data_ptr(), n, chunk), reps)
        ref = q[:n].clone()

        def host_cast():
            t0 = time.perf_counter()
            half[:n].copy_(src.t[:n])
            return 1e3 * (time.perf_counter() - t0)

        def move16(buf):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            q[:n].copy_(buf, non_blocking=True)
            torch.cuda.synchronize()
            return 1e3 * (time.perf_counter() - t0)

        def pageable():
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            q[:n].copy_(src.t[:n].to(torch.bfloat16))
            torch.cuda.synchronize()
            return 1e3 * (time.perf_counter() - t0)

        cast_ms = best_of(host_cast, reps)
        move_ms = best_of(lambda: move16(half[:n]), reps)
        assert torch.equal(q[:n].view(torch.int16), ref.view(torch.int16)), "the two routes disagree"
        page_ms = best_of(pageable, reps)
        rows.append({"fp32_bytes": 4 * n, "cast_on_gpu_move_fp32_ms": gpu_ms,
                     "cast_on_host_ms": cast_ms, "move_16bit_pinned_ms": move_ms,
                     "cast_on_host_move_16bit_ms": cast_ms + move_ms,
                     "cast_on_host_pageable_then_move_ms": page_ms,
                     "ratio_host_over_gpu": (cast_ms + move_ms) / gpu_ms})
        log(f"{4 * n / 2**20:7.0f} MB fp32: cast on GPU, move fp32 {gpu_ms:8.3f} ms ({4 * n / gpu_ms / 1e6:5.1f} GB/s)   "
            f"cast on host {cast_ms:8.3f} + move 16-bit {move_ms:8.3f} = {cast_ms + move_ms:8.3f} ms   "
            f"pageable route {page_ms:8.3f} ms   host/GPU {(cast_ms + move_ms) / gpu_ms:4.2f}x")
    B.so_destroy(ctx)
    src.free()
    half_store.free()
    print(json.dumps({"metric": "working_copy_from_host_fp32_ms", "unit": "ms", "n_gpus": 1, "data": "synthetic",
                      "config": {"workload": "fp32 parameters in pinned host memory, 1 MB ... 2 GB",
                                 "host_threads": threads, "chunk_elems": 1 << 24}, "rows": rows}), flush=True)


def speculative_bench(args):
    """Workload 2 (1.31 B parameters, 27 buckets of 50 M, fp16 gradients x loss scale): cost of
    one iteration under the three schedules, and of a rollback.
      synchronous   statistics pass, then one guarded multi-bucket step       30 B/param
      ping-pong     speculative step with by-product statistics, all buckets  28 B/param
                    in one launch (headline of this mode) or bucket by bucket
      save          per-bucket speculative step that also writes old p, m, v  40 B/param
    Rollback: ping-pong drops the alt set (pointer bookkeeping only); save copies p, m, v back
    and re-derives the working copy (26 B/param)."""
    import torch
    import synth
    from paper_2509_21271_amd import binding as B

    torch.cuda.set_device(0)
    dev = "cuda"
    cfg = synth.config(2)
    total = synth.total_params(2)
    bucket = cfg["bucket"]
    ranges = [(s, min(bucket, total - s)) for s in range(0, total, bucket)]
    scale = cfg["loss_scale"]
    ctx = B.so_create(0, torch.cuda.current_stream().cuda_stream)
    placement = {"arena_layout": args.arena_layout or "tuned"}
    if placement["arena_layout"] == "tuned":
        # both state sets inside one workspace, where the library's own timing of the ping-pong
        # step (both directions) finds them fastest; set-up, not timed
        factor = args.workspace_factor or 3.0
        ws_bytes = int(B.so_arena_plan(total).bytes * 1.75 * factor) // (2 << 20) * (2 << 20)
        t_tune = time.perf_counter()
        p, g, m, q, v, alt, arena_owner, tight_ms, tuned_ms = B.tuned_arena_views(
            ctx, total, torch.float16, ws_bytes, dev, trials=args.tune_trials, second_set=True)
        placement.update(workspace_gib=ws_bytes / 2**30, tune_s=time.perf_counter() - t_tune,
                         pingpong_kernel_ms_tight=tight_ms, pingpong_kernel_ms_tuned=tuned_ms)
        log(f"placement tuned in {placement['tune_s']:.1f} s inside {ws_bytes / 2**30:.1f} GiB: ping-pong step "
            f"{tight_ms:.3f} ms in the tight layout, {tuned_ms:.3f} ms where the arenas now lie")
    else:
        p = torch.empty(total, dtype=torch.float32, device=dev)
        m = torch.zeros(total, dtype=torch.float32, device=dev)
        v = torch.zeros(total, dtype=torch.float32, device=dev)
        q = torch.zeros(total, dtype=torch.bfloat16, device=dev)
        g = torch.empty(total, dtype=torch.float16, device=dev)
        alt = [torch.empty(total, dtype=torch.float32, device=dev) for _ in range(3)] + \
              [torch.zeros(total, dtype=torch.bfloat16, device=dev)]
    for s, n in ranges:
        p[s:s + n] = synth.normal_f32(cfg["seed"], synth.STREAM_PARAM, 0, s, n, cfg["sigma_p"], dev)
        g[s:s + n] = synth.normal_16bit(cfg["seed"], synth.STREAM_GRAD, 1, s, n, cfg["sigma_g"] * scale,
                                        torch.float16, dev)
    bks = [B.bucket_of(g[s:s + n], p[s:s + n], m[s:s + n], v[s:s + n], q[s:s + n], [a[s:s + n] for a in alt])
           for s, n in ranges]
    arr = (B.so_bucket * len(bks))(*bks)
    hp = B.hparams(cfg["hp"]["lr"], cfg["hp"]["beta1"], cfg["hp"]["beta2"], cfg["hp"]["eps"], cfg["hp"]["wd"])
    inv = 1.0 / scale
    nb = len(bks)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t0) / reps

    t = [1]

    def sync_iter():
        B.so_grad_stats_enqueue(ctx, arr, scale, 0.0)
        B.so_adam_step_guarded(ctx, arr, hp, t[0])
        t[0] += 1

    def spec_iter(mode, resolve):
        for k in range(nb):
            B.so_adam_step(ctx, arr[k], hp, t[0], inv, mode)
        st = B.so_adam_step_stats(ctx)
        dec = B.so_validate(st, 0.0, scale, 1.0)
        assert dec.action == B.SO_COMMIT
        for k in range(nb):
            resolve(ctx, arr[k])
        t[0] += 1

    def spec_multi_iter(mode, resolve):
        """All buckets' gradients ready: ONE speculative launch over the bucket list."""
        B.so_adam_step_multi(ctx, arr, hp, t[0], inv, mode)
        st = B.so_adam_step_stats(ctx)
        dec = B.so_validate(st, 0.0, scale, 1.0)
        assert dec.action == B.SO_COMMIT
        for k in range(nb):
            resolve(ctx, arr[k])
        t[0] += 1

    def redo_iter(mode):
        """Validation says "clipped": roll the speculative step back, run it again with the
        clipped multiplier in one multi-bucket launch (Sec. 4.4, scenario 2)."""
        for k in range(nb):
            B.so_adam_step(ctx, arr[k], hp, t[0], inv, mode)
        st = B.so_adam_step_stats(ctx)
        dec = B.so_validate(st, 1.0, scale, 1.0)
        assert dec.action == B.SO_ROLLBACK_REDO
        for k in range(nb):
            B.so_adam_rollback(ctx, arr[k])
        B.so_adam_step_multi(ctx, arr, hp, t[0], dec.grad_scale)
        t[0] += 1

    reps = args.steps
    res = {"synchronous_ms": timed(sync_iter, reps),
           "pingpong_commit_ms": timed(lambda: spec_iter(B.SO_SPEC_PINGPONG, B.so_adam_commit), reps),
           "pingpong_one_launch_commit_ms": timed(lambda: spec_multi_iter(B.SO_SPEC_PINGPONG, B.so_adam_commit), reps),
           "save_commit_ms": timed(lambda: spec_iter(B.SO_SPEC_SAVE, B.so_adam_commit), reps),
           "pingpong_rollback_iter_ms": timed(lambda: spec_iter(B.SO_SPEC_PINGPONG, B.so_adam_rollback), reps),
           "save_rollback_iter_ms": timed(lambda: spec_iter(B.SO_SPEC_SAVE, B.so_adam_rollback), reps),
           "pingpong_redo_iter_ms": timed(lambda: redo_iter(B.SO_SPEC_PINGPONG), reps),
           "save_redo_iter_ms": timed(lambda: redo_iter(B.SO_SPEC_SAVE), reps)}
    res["pingpong_rollback_ms"] = res["pingpong_rollback_iter_ms"] - res["pingpong_commit_ms"]
    res["save_rollback_ms"] = res["save_rollback_iter_ms"] - res["save_commit_ms"]
    B.so_destroy(ctx)
    out = {"metric": "adam_speculative_iteration_ms", "value": res["pingpong_one_launch_commit_ms"], "unit": "ms",
           "n_gpus": 1, "steps": reps, "warmup": 1, "ms_per_step": res["pingpong_one_launch_commit_ms"],
           "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
           "data": "synthetic",
           "config": {"workload": cfg["name"], "params": total, "buckets": nb, "bucket_elems": bucket,
                      "grad_dtype": "fp16", "loss_scale": scale, "placement": placement},
           "schedules": {k: round(x, 3) for k, x in res.items()},
           "gbps": {"synchronous": 30 * total / res["synchronous_ms"] / 1e6,
                    "pingpong": 28 * total / res["pingpong_commit_ms"] / 1e6,
                    "pingpong_one_launch": 28 * total / res["pingpong_one_launch_commit_ms"] / 1e6,
                    "save": 40 * total / res["save_commit_ms"] / 1e6}}
    print(json.dumps(out), flush=True)


def overlap_bench(args):
    """Workload 2 under a stand-in backward pass: what speculation-then-validation is for
    (Sec. 4.4).  Bucket k's gradients "arrive" when a compute-bound stand-in for its share of
    the backward pass (library bf16 GEMMs on a second stream -- plumbing of this benchmark, not
    part of the library) has finished.
      synchronous   every step waits for the last gradient: backward, then statistics + step
      speculative   bucket k is stepped (ping-pong, statistics as a by-product) as soon as its
                    gradients exist, under the backward pass of the buckets still to come;
                    after the last one: validation, commit
    Reported: iteration time of both, the backward stand-in alone, and the optimizer time each
    schedule leaves exposed."""
    import torch
    import synth
    from paper_2509_21271_amd import binding as B

    torch.cuda.set_device(0)
    dev = "cuda"
    cfg = synth.config(2)
    total = synth.total_params(2)
    bucket = cfg["bucket"]
    ranges = [(s, min(bucket, total - s)) for s in range(0, total, bucket)]
    scale = cfg["loss_scale"]
    p = torch.empty(total, dtype=torch.float32, device=dev)
    m = torch.zeros(total, dtype=torch.float32, device=dev)
    v = torch.zeros(total, dtype=torch.float32, device=dev)
    q = torch.zeros(total, dtype=torch.bfloat16, device=dev)
    g = torch.empty(total, dtype=torch.float16, device=dev)
    alt = [torch.empty(total, dtype=torch.float32, device=dev) for _ in range(3)] + \
          [torch.zeros(total, dtype=torch.bfloat16, device=dev)]
    for s0, n in ranges:
        p[s0:s0 + n] = synth.normal_f32(cfg["seed"], synth.STREAM_PARAM, 0, s0, n, cfg["sigma_p"], dev)
        g[s0:s0 + n] = synth.normal_16bit(cfg["seed"], synth.STREAM_GRAD, 1, s0, n, cfg["sigma_g"] * scale,
                                          torch.float16, dev)
    bks = [B.bucket_of(g[s0:s0 + n], p[s0:s0 + n], m[s0:s0 + n], v[s0:s0 + n], q[s0:s0 + n],
                       [a[s0:s0 + n] for a in alt]) for s0, n in ranges]
    arr = (B.so_bucket * len(bks))(*bks)
    main = torch.cuda.current_stream()
    ctx = B.so_create(0, main.cuda_stream)
    hp = B.hparams(cfg["hp"]["lr"], cfg["hp"]["beta1"], cfg["hp"]["beta2"], cfg["hp"]["eps"], cfg["hp"]["wd"])
    nb = len(bks)
    inv = 1.0 / scale

    # the stand-in: GEMMs of 4096^3, as many per bucket as fill --bwd-ms-per-bucket
    bwd = torch.cuda.Stream()
    a = torch.randn(4096, 4096, dtype=torch.bfloat16, device=dev)
    b = torch.randn(4096, 4096, dtype=torch.bfloat16, device=dev)
    c = torch.empty(4096, 4096, dtype=torch.bfloat16, device=dev)
    for _ in range(5):
        torch.matmul(a, b, out=c)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(50):
        torch.matmul(a, b, out=c)
    torch.cuda.synchronize()
    gemm_ms = 1e3 * (time.perf_counter() - t0) / 50
    per_bucket = max(1, round(args.bwd_ms_per_bucket / gemm_ms))
    log(f"stand-in GEMM {gemm_ms:.3f} ms ({2 * 4096 ** 3 / gemm_ms / 1e9:.0f} TFLOP/s), {per_bucket} per bucket")
    events = [torch.cuda.Event() for _ in range(nb)]

    def backward(k):
        with torch.cuda.stream(bwd):
            for _ in range(per_bucket):
                torch.matmul(a, b, out=c)
            events[k].record(bwd)

    t = [1]

    def backward_only():
        bwd.wait_stream(main)
        for k in range(nb):
            backward(k)
        main.wait_event(events[nb - 1])

    def synchronous():
        bwd.wait_stream(main)
        for k in range(nb):
            backward(k)
        main.wait_event(events[nb - 1])
        B.so_grad_stats_enqueue(ctx, arr, scale, 0.0)
        B.so_adam_step_guarded(ctx, arr, hp, t[0])
        st, dec = B.so_grad_stats_fetch(ctx)
        assert dec.action == B.SO_COMMIT
        t[0] += 1

    def speculative():
        bwd.wait_stream(main)
        for k in range(nb):
            backward(k)
            main.wait_event(events[k])
            B.so_adam_step(ctx, arr[k], hp, t[0], inv, B.SO_SPEC_PINGPONG)
        st = B.so_adam_step_stats(ctx)
        dec = B.so_validate(st, 0.0, scale, 1.0)
        assert dec.action == B.SO_COMMIT
        for k in range(nb):
            B.so_adam_commit(ctx, arr[k])
        t[0] += 1

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
            torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t0) / reps

    reps = args.steps
    res = {"backward_only_ms": timed(backward_only, reps),
           "synchronous_ms": timed(synchronous, reps),
           "speculative_ms": timed(speculative, reps)}
    res["exposed_optimizer_ms_synchronous"] = res["synchronous_ms"] - res["backward_only_ms"]
    res["exposed_optimizer_ms_speculative"] = res["speculative_ms"] - res["backward_only_ms"]
    B.so_destroy(ctx)
    out = {"metric": "adam_exposed_optimizer_ms", "value": res["exposed_optimizer_ms_speculative"], "unit": "ms",
           "n_gpus": 1, "steps": reps, "warmup": 1, "ms_per_step": res["speculative_ms"],
           "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": cfg["name"], "params": total, "buckets": nb, "bucket_elems": bucket,
                      "backward_stand_in": f"{per_bucket} bf16 GEMMs of 4096^3 per bucket on a second stream "
                                           f"({gemm_ms:.3f} ms each alone)"},
           "schedules": {k: round(x, 3) for k, x in res.items()}}
    print(json.dumps(out), flush=True)


def latency_table(args):
    """Step latency at the parameter counts of the paper's Adam latency table (Sec. 5.6:
    1, 2, 4, 8 billion parameters), step kernel alone (28 B/param), 100 M-element buckets in
    one launch.  The paper's GraceAdam column (72-core Grace CPU) is printed beside it as
    context: another machine, another memory system."""
    import torch
    import synth
    from paper_2509_21271_amd import binding as B

    torch.cuda.set_device(0)
    cfg = synth.config(3)
    bucket = cfg["bucket"]
    hp = B.hparams(cfg["hp"]["lr"], cfg["hp"]["beta1"], cfg["hp"]["beta2"], cfg["hp"]["eps"], cfg["hp"]["wd"])
    paper_graceadam_s = {1: 0.082, 2: 0.160, 4: 0.316, 8: 0.608}
    top = 8_000_000_000
    p = torch.empty(top, dtype=torch.float32, device="cuda")
    m = torch.zeros(top, dtype=torch.float32, device="cuda")
    v = torch.zeros(top, dtype=torch.float32, device="cuda")
    q = torch.zeros(top, dtype=torch.bfloat16, device="cuda")
    g = torch.empty(top, dtype=torch.bfloat16, device="cuda")
    for s0 in range(0, top, bucket):
        p[s0:s0 + bucket] = synth.normal_f32(cfg["seed"], synth.STREAM_PARAM, 0, s0, bucket, cfg["sigma_p"], "cuda")
        g[s0:s0 + bucket] = synth.normal_16bit(cfg["seed"], synth.STREAM_GRAD, 1, s0, bucket, cfg["sigma_g"],
                                               torch.bfloat16, "cuda")
    ctx = B.so_create(0, torch.cuda.current_stream().cuda_stream)
    rows = []
    t_adam = 1
    for billions in (1, 2, 4, 8):
        n = billions * 1_000_000_000
        bs = [B.bucket_of(g[s0:s0 + bucket], p[s0:s0 + bucket], m[s0:s0 + bucket], v[s0:s0 + bucket],
                          q[s0:s0 + bucket]) for s0 in range(0, n, bucket)]
        arr = (B.so_bucket * len(bs))(*bs)
        for _ in range(args.warmup):
            B.so_adam_step_multi(ctx, arr, hp, t_adam, 0.01)
            t_adam += 1
        B.so_set_profiling(ctx, True)
        for _ in range(args.steps):
            B.so_adam_step_multi(ctx, arr, hp, t_adam, 0.01)
            t_adam += 1
        ms = B.so_read_step_kernel_ms(ctx)
        B.so_set_profiling(ctx, False)
        med = sorted(ms)[len(ms) // 2]
        rows.append({"params": n, "ms_median": med, "ms_min": min(ms),
                     "gbps": STEP_BYTES_PER_PARAM * n / (med * 1e-3) / 1e9,
                     "paper_graceadam_ms_other_machine": 1e3 * paper_graceadam_s[billions]})
        log(f"{billions} B params: {med:.3f} ms  {rows[-1]['gbps']:.0f} GB/s   (paper, Grace CPU: "
            f"{1e3 * paper_graceadam_s[billions]:.0f} ms)")
    B.so_destroy(ctx)
    print(json.dumps({"metric": "adam_step_latency_ms", "unit": "ms", "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "higher_is_better": False, "dtype": "f32", "data": "synthetic",
                      "vs_baseline": None, "config": {"workload": "flat state of 1/2/4/8 billion parameters, "
                                                      "100 M-element buckets, step kernel alone"},
                      "rows": rows}), flush=True)


def _event_ms(fn, reps, warm=2):
    """Median / min duration of fn() in ms, by HIP events on torch's current stream (the stream
    the context launches on)."""
    import torch
    for _ in range(warm):
        fn()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in ev)
    return ms[len(ms) // 2], ms[0]


def ceilings_bench(args):
    """What the chip sustains through the library's own kernels, on one box in one process: a
    plain copy and a copy with statistics (flatten_kernel), the read-only statistics pass
    (grad_stats_kernel), the restore pass of a save-mode rollback (restore_kernel), and the
    step kernel in place, out of place (ping-pong) and in save mode.  2 x 10^9 parameters of flat
    state; algorithmic bytes per element as listed.  These are the same-box reference rates the
    step kernel's roofline fraction is read against."""
    import torch
    import synth
    from paper_2509_21271_amd import binding as B

    torch.cuda.set_device(0)
    dev = "cuda"
    n = 2_000_000_000        # not a power of two: arrays a power of two apart would alias in the memory channels
    cfg = synth.config(3)
    hp = B.hparams(cfg["hp"]["lr"], cfg["hp"]["beta1"], cfg["hp"]["beta2"], cfg["hp"]["eps"], cfg["hp"]["wd"])
    p = torch.empty(n, dtype=torch.float32, device=dev)
    chunk = 100_000_000
    for s0 in range(0, n, chunk):
        p[s0:s0 + chunk] = synth.normal_f32(cfg["seed"], synth.STREAM_PARAM, 0, s0, chunk, cfg["sigma_p"], dev)
    m = torch.zeros(n, dtype=torch.float32, device=dev)
    v = torch.zeros(n, dtype=torch.float32, device=dev)
    q = torch.zeros(n, dtype=torch.bfloat16, device=dev)
    g = torch.empty(n, dtype=torch.bfloat16, device=dev)
    for s0 in range(0, n, chunk):
        g[s0:s0 + chunk] = synth.normal_16bit(cfg["seed"], synth.STREAM_GRAD, 1, s0, chunk, cfg["sigma_g"],
                                              torch.bfloat16, dev)
    alt = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(3)] + \
          [torch.zeros(n, dtype=torch.bfloat16, device=dev)]
    g2 = torch.empty(n, dtype=torch.bfloat16, device=dev)
    ctx = B.so_create(0, torch.cuda.current_stream().cuda_stream)
    bk = B.bucket_of(g, p, m, v, q, alt)
    one = B.so_slice(0, 0, 0, 0, n)
    t = [1]
    reps = args.steps

    def step(mode):
        B.so_adam_step(ctx, bk, hp, t[0], 0.01, mode)
        if mode != B.SO_SYNC:
            B.so_adam_commit(ctx, bk)
        t[0] += 1

    def save_then_restore():
        B.so_adam_step(ctx, bk, hp, t[0], 0.01, B.SO_SPEC_SAVE)
        B.so_adam_rollback(ctx, bk)

    rows = []

    def row(name, kernel, bytes_per_elem, fn, minus_ms=0.0):
        med, mn = _event_ms(fn, reps)
        med -= minus_ms
        rows.append({"what": name, "kernel": kernel, "bytes_per_elem": bytes_per_elem, "ms_median": med,
                     "gbps": bytes_per_elem * n / (med * 1e-3) / 1e9,
                     "frac_of_peak": bytes_per_elem * n / (med * 1e-3) / 1e9 / HBM_PEAK_GBPS})
        log(f"{name:58s} {med:8.3f} ms  {rows[-1]['gbps']:7.0f} GB/s  {100 * rows[-1]['frac_of_peak']:.1f} %")
        return med

    row("copy, fp32 (4 B read + 4 B written)", "flatten_kernel<unsigned int, -1>", 8,
        lambda: B.so_flatten(ctx, [one], [p.data_ptr()], [alt[0].data_ptr()], 4, 0))
    row("copy, 16 bit (2 B read + 2 B written)", "flatten_kernel<unsigned short, -1>", 4,
        lambda: B.so_flatten(ctx, [one], [g.data_ptr()], [g2.data_ptr()], 2, 0))
    off1 = B.so_slice(0, 1, 0, 0, n - 8)      # the source starts one element past a 16-byte boundary
    row("copy, 16 bit, source 2 bytes off its 16-byte granule", "flatten_kernel<unsigned short, -1>", 4,
        lambda: B.so_flatten(ctx, [off1], [g.data_ptr()], [g2.data_ptr()], 2, 0))
    row("copy, fp32, source 4 bytes off its 16-byte granule", "flatten_kernel<unsigned int, -1>", 8,
        lambda: B.so_flatten(ctx, [off1], [p.data_ptr()], [alt[0].data_ptr()], 4, 0))
    row("copy + gradient statistics, 16 bit (2 B read + 2 B written)", "flatten_kernel<unsigned short, 0>", 4,
        lambda: B.so_flatten_grad_stats(ctx, [one], [g.data_ptr()], [g2.data_ptr()], B.SO_GRAD_BF16, 1.0, 1.0))
    row("working copy from fp32 parameters (4 B read + 2 B written)", "cast_lp_kernel", 6,
        lambda: B.so_cast_params(ctx, p.data_ptr(), alt[3].data_ptr(), n))
    row("gradient statistics, read only (2 B read)", "grad_stats_kernel<0>", 2,
        lambda: B.so_grad_stats_enqueue(ctx, bk, 1.0, 1.0))
    sync_ms = row("step in place (14 B read + 14 B written)", "adam_step_kernel<0, 0, true>", 28,
                  lambda: step(B.SO_SYNC))
    row("step out of place, ping-pong (14 B read + 14 B written)", "adam_step_kernel<0, 1, true>", 28,
        lambda: step(B.SO_SPEC_PINGPONG))
    B.so_adam_step_stats(ctx)
    save_ms = row("step in save mode (14 B read + 26 B written)", "adam_step_kernel<0, 2, true>", 40,
                  lambda: step(B.SO_SPEC_SAVE))
    B.so_adam_step_stats(ctx)
    row("restore after a save-mode step (12 B read + 14 B written)", "restore_kernel", 26, save_then_restore,
        minus_ms=save_ms)
    B.so_adam_step_stats(ctx)
    B.so_destroy(ctx)
    print(json.dumps({"metric": "product_kernel_bandwidth_gbps", "unit": "GB/s", "n_gpus": 1, "steps": reps,
                      "data": "synthetic", "dtype": "f32", "vs_baseline": None,
                      "config": {"workload": f"flat state of {n} parameters, one bucket"},
                      "peak": HBM_PEAK_GBPS, "rows": rows}), flush=True)


def flatten_bench(args):
    """Workload 3 with gradients arriving as per-tensor arrays (291 tensors): gather into the
    81 buckets, validate, step.  Two schedules of the same work:
      separate   so_flatten, so_grad_stats_enqueue, so_adam_step_guarded     4 + 2 + 28 B/param
      fused      so_flatten_grad_stats, so_adam_step_guarded                 4 + 28 B/param"""
    import torch
    import synth
    from paper_2509_21271_amd import binding as B

    torch.cuda.set_device(0)
    dev = "cuda"
    cfg = synth.config(3)
    total = synth.total_params(3)
    bucket = cfg["bucket"]
    ranges = [(s, min(bucket, total - s)) for s in range(0, total, bucket)]
    numel = [k for _, k in synth.tensor_list(3)]
    slices, nb = B.so_layout_plan(numel, bucket)
    p, g, m, q, v, (src,), arena_owner = B.arena_views(total, torch.bfloat16, dev, extra_16bit=1)
    g.zero_()                                                         # src: the per-tensor gradient arrays
    for s, n in ranges:
        p[s:s + n] = synth.normal_f32(cfg["seed"], synth.STREAM_PARAM, 0, s, n, cfg["sigma_p"], dev)
    offs = [0]
    for k in numel:
        offs.append(offs[-1] + k)
    tptr = [src.data_ptr() + 2 * o for o in offs[:-1]]
    bptr = [g.data_ptr() + 2 * s for s, _ in ranges]
    buckets = [B.bucket_of(g[s:s + n], p[s:s + n], m[s:s + n], v[s:s + n], q[s:s + n]) for s, n in ranges]
    arr = (B.so_bucket * len(buckets))(*buckets)
    ctx = B.so_create(0, torch.cuda.current_stream().cuda_stream)
    hp = B.hparams(cfg["hp"]["lr"], cfg["hp"]["beta1"], cfg["hp"]["beta2"], cfg["hp"]["eps"], cfg["hp"]["wd"])
    t = [1]

    def fresh():
        for s, n in ranges:
            src[s:s + n] = synth.normal_16bit(cfg["seed"], synth.STREAM_GRAD, t[0], s, n, cfg["sigma_g"],
                                              torch.bfloat16, dev)

    def separate():
        B.so_flatten(ctx, slices, tptr, bptr, 2, 0)
        B.so_grad_stats_enqueue(ctx, arr, 1.0, cfg["max_norm"])
        B.so_adam_step_guarded(ctx, arr, hp, t[0])

    def fused():
        B.so_flatten_grad_stats(ctx, slices, tptr, bptr, B.SO_GRAD_BF16, 1.0, cfg["max_norm"])
        B.so_adam_step_guarded(ctx, arr, hp, t[0])

    res = {}
    for name, fn in (("separate", separate), ("fused", fused)):
        wall = 0.0
        for k in range(args.warmup + args.steps):
            fresh()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            if k >= args.warmup:
                wall += time.perf_counter() - t0
            t[0] += 1
        res[name] = 1e3 * wall / args.steps
        st, dec = B.so_grad_stats_fetch(ctx)
        log(f"{name}: {res[name]:.3f} ms per step (norm {st.norm:.4f}, clip {dec.clip:.6f})")
    gather_ms = _event_ms(lambda: B.so_flatten(ctx, slices, tptr, bptr, 2, 0), args.steps)[0]
    gather_stats_ms = _event_ms(lambda: B.so_flatten_grad_stats(ctx, slices, tptr, bptr, B.SO_GRAD_BF16, 1.0,
                                                                 cfg["max_norm"]), args.steps)[0]
    B.so_destroy(ctx)
    print(json.dumps({"metric": "adam_step_params_per_s", "value": total / (res["fused"] * 1e-3), "unit": "params/s",
                      "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["fused"],
                      "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
                      "data": "synthetic",
                      "config": {"workload": cfg["name"], "params": total, "buckets": len(ranges),
                                 "gradient_tensors": len(numel), "slices": len(slices),
                                 "schedule": "gather with fused statistics + GPU-side validation + guarded step"},
                      "ms_per_step_separate_statistics": res["separate"],
                      "gather_ms": gather_ms, "gather_with_statistics_ms": gather_stats_ms,
                      "gather_gbps": 4 * total / (gather_ms * 1e-3) / 1e9,
                      "gather_with_statistics_gbps": 4 * total / (gather_stats_ms * 1e-3) / 1e9}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, help="workload (default 3: Llama-3-8B-shaped)")
    ap.add_argument("--layers", type=int, default=7,
                    help="workload 4 only: layers kept (48 = full size, needs 280 GB pinned host memory)")
    ap.add_argument("--resident-buckets", type=int, default=0,
                    help="with --config 4: this many extra buckets stay on the GPU (so_hybrid_step)")
    ap.add_argument("--unpinned", action="store_true",
                    help="with --config 4: keep the host state in pageable memory (comparison only)")
    ap.add_argument("--plan", action="store_true",
                    help="workload 4 only: measured move/step times and the resident-bucket count they imply")
    ap.add_argument("--bucket-sweep", action="store_true",
                    help="workload 4 only: host-link rate versus staged bucket size")
    ap.add_argument("--cast-variants", action="store_true",
                    help="with --config 4: working copy from host fp32 parameters, cast on the GPU "
                         "(move fp32) against cast on the host (move 16 bits), 1 MB ... 2 GB (Sec. 4.5)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--ceilings", action="store_true",
                    help="bandwidth of the library's own kernels (copy, statistics, restore, step variants) "
                         "on 2 x 10^9 parameters: the same-box reference rates")
    ap.add_argument("--flatten", action="store_true",
                    help="workload 3 with per-tensor gradient arrays: gather + statistics fused versus separate")
    ap.add_argument("--workspace-factor", type=float, default=None,
                    help="with --arena-layout tuned: size of the workspace as a multiple of the state's size "
                         "(default 1.5; 3 for --config 2)")
    ap.add_argument("--tune-trials", type=int, default=60,
                    help="with --arena-layout tuned: random placements so_arena_tune times")
    ap.add_argument("--arena-layout", choices=["one-allocation", "five-allocations", "tuned"], default=None,
                    help="default workloads: the five flat arenas in one device allocation, ordered p g m q v "
                         "(default), as five allocations, or inside a larger workspace where so_arena_tune "
                         "finds the step fastest; --config 2: tuned (default) or anything else for nine "
                         "separate allocations")
    ap.add_argument("--separate-buckets", action="store_true",
                    help="default workloads: allocate every bucket's arrays separately, so that the step "
                         "runs through the bucket table instead of one merged range")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain copy of 2^28 fp32 elements (1 GiB read + 1 GiB written, "
                         "flatten_kernel) as the known-size reference for rocprofv3 byte counters")
    ap.add_argument("--overlap", action="store_true",
                    help="with --config 2: speculative steps under a stand-in backward pass")
    ap.add_argument("--bwd-ms-per-bucket", type=float, default=1.0,
                    help="with --overlap: length of the stand-in backward pass per bucket")
    ap.add_argument("--latency-table", action="store_true",
                    help="step latency at 1, 2, 4, 8 billion parameters (the sizes of the paper's Adam "
                         "latency table)")
    ap.add_argument("--graph", action="store_true",
                    help="record one autonomous iteration as a HIP graph and replay it per step")
    ap.add_argument("--autonomous", action="store_true",
                    help="one so_train_iteration per step: step count, loss scale and validation stay on the GPU")
    ap.add_argument("--host-validated", action="store_true",
                    help="use so_grad_stats + so_validate on the host instead of the guarded step")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (the path has no inter-GPU part); "
                 "use --gpus 1")

    import torch
    import synth
    from paper_2509_21271_amd import binding as B

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.latency_table:
        return latency_table(args)
    if args.ceilings:
        return ceilings_bench(args)
    if args.flatten:
        return flatten_bench(args)
    if args.config == 4 and args.plan:
        return repartition_plan(args)
    if args.config == 4 and args.bucket_sweep:
        return bucket_sweep(args)
    if args.config == 4 and args.cast_variants:
        return cast_variants(args)
    if args.config == 4:
        return stream_bench(args)
    if args.config == 2 and args.overlap:
        return overlap_bench(args)
    if args.config == 2:
        return speculative_bench(args)
    torch.cuda.set_device(0)
    dev = "cuda"
    cfg = synth.config(args.config)
    total = synth.total_params(args.config)
    bucket = cfg["bucket"]
    gdt = torch.float16 if cfg["grad_dtype"] == "fp16" else torch.bfloat16
    ranges = [(s, min(bucket, total - s)) for s in range(0, total, bucket)]
    log(f"workload {cfg['name']}: {total} params, {len(ranges)} buckets of {bucket}")

    args.arena_layout = args.arena_layout or "one-allocation"
    if args.separate_buckets:
        # every bucket's five arrays are allocations of their own (with a gap, so that no two are
        # adjacent): the step then runs through the device bucket table, not one merged range
        views, gaps = [], []
        for s, n in ranges:
            one = []
            for dt in (gdt, torch.float32, torch.float32, torch.float32, torch.bfloat16):
                one.append(torch.zeros(n, dtype=dt, device=dev))
                gaps.append(torch.empty(4096, dtype=torch.uint8, device=dev))
            one[1].copy_(synth.normal_f32(cfg["seed"], synth.STREAM_PARAM, 0, s, n, cfg["sigma_p"], dev))
            views.append(one)
    else:
        # flat arenas, one per array kind; a bucket is the same index range in all five
        if args.arena_layout == "tuned":
            # a workspace larger than the state; the library times its own step kernel on candidate
            # placements of the five arenas inside it and keeps the fastest (set-up, not timed)
            tune_ctx = B.so_create(0, torch.cuda.current_stream().cuda_stream)
            ws_bytes = int(B.so_arena_plan(total).bytes * (args.workspace_factor or 1.5)) // (2 << 20) * (2 << 20)
            t_tune = time.perf_counter()
            p, g, m, q, v, _, arena_owner, tight_ms, tuned_ms = B.tuned_arena_views(
                tune_ctx, total, gdt, ws_bytes, dev, trials=args.tune_trials)
            B.so_destroy(tune_ctx)
            log(f"placement tuned in {time.perf_counter() - t_tune:.1f} s inside {ws_bytes / 2**30:.1f} GiB: "
                f"step kernel {tight_ms:.3f} ms in the tight layout, {tuned_ms:.3f} ms where the arenas now lie")
        elif args.arena_layout == "one-allocation":
            # ONE device allocation, arenas in the order the library recommends (so_arena_plan):
            # p g m q v, the way a trainer that sets its state up once at start-up would do
            p, g, m, q, v, _, arena_owner = B.arena_views(total, gdt, dev)
        else:
            p = torch.empty(total, dtype=torch.float32, device=dev)
            m = torch.zeros(total, dtype=torch.float32, device=dev)
            v = torch.zeros(total, dtype=torch.float32, device=dev)
            q = torch.zeros(total, dtype=torch.bfloat16, device=dev)
            g = torch.empty(total, dtype=gdt, device=dev)
        for s, n in ranges:
            p[s:s + n] = synth.normal_f32(cfg["seed"], synth.STREAM_PARAM, 0, s, n, cfg["sigma_p"], dev)
        views = [[g[s:s + n], p[s:s + n], m[s:s + n], v[s:s + n], q[s:s + n]] for s, n in ranges]
    buckets = [B.bucket_of(*vw) for vw in views]
    arr = (B.so_bucket * len(buckets))(*buckets)

    ctx = B.so_create(0, torch.cuda.current_stream().cuda_stream)
    hp = B.hparams(cfg["hp"]["lr"], cfg["hp"]["beta1"], cfg["hp"]["beta2"], cfg["hp"]["eps"], cfg["hp"]["wd"])
    loss_scale = cfg["loss_scale"]

    def fresh_grads(step):
        for (s, n), vw in zip(ranges, views):
            vw[0].copy_(synth.normal_16bit(cfg["seed"], synth.STREAM_GRAD, step, s, n,
                                           cfg["sigma_g"] * loss_scale, gdt, dev))

    if args.graph:
        args.autonomous = True
    if args.autonomous:
        B.so_train_reset(ctx, hp, 1, loss_scale, 1.0, 2.0 ** 24, 0, cfg["max_norm"])
    if args.graph:
        B.so_train_capture(ctx, arr)

    def one_step(t):
        if args.graph:
            B.so_train_replay(ctx)
        elif args.autonomous:
            B.so_train_iteration(ctx, arr)
        elif args.host_validated:
            st = B.so_grad_stats(ctx, arr, 1.0 / loss_scale)
            dec = B.so_validate(st, cfg["max_norm"], loss_scale, 1.0)
            if dec.action != B.SO_ROLLBACK_SKIP:
                B.so_adam_step_multi(ctx, arr, hp, t, dec.grad_scale)
        else:
            B.so_grad_stats_enqueue(ctx, arr, loss_scale, cfg["max_norm"])
            B.so_adam_step_guarded(ctx, arr, hp, t)

    t_adam = 1
    for w in range(args.warmup):
        fresh_grads(t_adam)
        one_step(t_adam)
        t_adam += 1
    torch.cuda.synchronize()

    B.so_set_profiling(ctx, True)
    wall = 0.0
    enqueue_s = 0.0
    for k in range(args.steps):
        fresh_grads(t_adam)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        one_step(t_adam)
        t_enq = time.perf_counter()
        torch.cuda.synchronize()
        wall += time.perf_counter() - t0
        enqueue_s += t_enq - t0
        t_adam += 1
    kernel_ms = B.so_read_step_kernel_ms(ctx)
    B.so_set_profiling(ctx, False)
    if args.calibrate_copy:
        n_cal = 1 << 28
        src = torch.ones(n_cal, dtype=torch.float32, device=dev)
        dst = torch.zeros(n_cal, dtype=torch.float32, device=dev)
        sl = B.so_slice(0, 0, 0, 0, n_cal)
        B.so_flatten(ctx, [sl], [src.data_ptr()], [dst.data_ptr()], 4, 0)
        torch.cuda.synchronize()
        assert bool((dst == 1).all())
        del src, dst
    if args.autonomous:
        st, dec, applied, _ = B.so_train_fetch(ctx)
        assert applied == args.warmup + args.steps
    else:
        st, dec = (B.so_grad_stats_fetch(ctx) if not args.host_validated else (None, None))
    if args.graph:          # launches inside a recorded graph carry no event pairs
        kernel_ms = [wall * 1e3 / args.steps]
    assert len(kernel_ms) == (1 if args.graph else args.steps), (len(kernel_ms), args.steps)

    ms_per_step = wall * 1e3 / args.steps
    k_avg = sum(kernel_ms) / len(kernel_ms)
    kernel_bytes = (STEP_BYTES_PER_PARAM + STATS_BYTES_PER_PARAM) if args.graph else STEP_BYTES_PER_PARAM
    achieved = kernel_bytes * total / (k_avg * 1e-3) / 1e9
    out = {
        "metric": "adam_step_params_per_s",
        "value": total / (ms_per_step * 1e-3),
        "unit": "params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": cfg["name"], "params": total, "buckets": len(ranges),
                   "bucket_elems": bucket, "grad_dtype": cfg["grad_dtype"], "max_norm": cfg["max_norm"],
                   "bucket_memory": "separate allocations (bucket-table launch)" if args.separate_buckets else
                                    "flat arenas (adjacent buckets merge into one range), " + args.arena_layout,
                   "schedule": "host-validated" if args.host_validated else
                               "autonomous, replayed from a HIP graph" if args.graph else
                               "autonomous (step count, loss scale, validation on the GPU)" if args.autonomous else
                               "grad-stats + GPU-side validation + guarded fused step",
                   },
        "gparams_per_s": total / (ms_per_step * 1e-3) / 1e9,
        "step_gbps_whole_path": (STEP_BYTES_PER_PARAM + STATS_BYTES_PER_PARAM) * total / (ms_per_step * 1e-3) / 1e9,
        "host_enqueue_ms_per_step": enqueue_s * 1e3 / args.steps,
        "roofline": {"bound": "hbm", "kernel": "whole recorded iteration (statistics + validation + step, 30 B/param)"
                     if args.graph else "adam_step_kernel (fused AdamW + bf16 cast, all buckets, one launch)",
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": measured_traffic(f"adam_step_kernel_config{args.config}_pmc.txt"),
                     "traffic_source": f"profiles/adam_step_kernel_config{args.config}_pmc.txt (rocprofv3 --pmc "
                                       "FETCH_SIZE / WRITE_SIZE runs of the same launch; not measured in this run)",
                     "algorithmic_bytes_per_launch": kernel_bytes * total,
                     "kernel_ms_avg": k_avg, "kernel_ms_min": min(kernel_ms),
                     "kernel_ms_median": sorted(kernel_ms)[len(kernel_ms) // 2]},
    }
    if st is not None:
        out["config"]["last_norm"] = st.norm
        out["config"]["last_clip"] = dec.clip
    if not args.no_cpu_baseline:
        # the GPU machines give one job 16 host threads whatever os.cpu_count() says
        threads = min(16, os.cpu_count() or 1)
        sample = min(total, 1 << 28)
        out["cpu_baseline"] = cpu_baseline(cfg, total, bucket, t_adam, threads, sample)
        one = cpu_baseline(cfg, total, bucket, t_adam, 1, min(total, 1 << 25))
        out["cpu_baseline"]["single_thread"] = {"value": one["value"], "unit": one["unit"], "sample": one["sample"]}
        out["cpu_baseline"]["host_cores_visible"] = os.cpu_count()
        out["cpu_baseline"]["threads_note"] = "cores = host threads the oracle ran on (this pool grants a job 16)"
    B.so_destroy(ctx)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
