#!/usr/bin/env python3
"""Benchmark of the APAR decode path on one MI355X.

A step is one pass of the whole hot path over the live threads of a synthetic fork-tree
workload: a few threads finish and a forked child carries on in their place (apar_fork +
apar_free_thread), every live thread appends the new token's K,V row (apar_append_kv_batch,
with copy-on-write where a tail is shared), and all live threads attend over their root
paths (apar_decode_attention).  Inputs are resident in HBM before the timed region.

Prints ONE JSON line: metric, value, unit, the step counts and times, `roofline` (the attention kernel's
algorithmic bytes over its measured duration against the HBM peak), `cpu_baseline` (the oracle timed on the host),
a breakdown of the step, the KV bytes resident, and the other configurations under `secondary`.
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

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak


def _oracle_requests(task):
    """Worker of the cpu_baseline leg (its own process: numpy and the oracle only, one BLAS thread).
    Decodes one step for every live thread of the given requests of a workload with the fp64 oracle as it
    stands; returns (pid, threads, attended tokens, seconds decoding, seconds materialising the copies)."""
    w_name, seed, n_req, requests = task
    import numpy as np  # noqa: F401
    from threadpoolctl import threadpool_limits

    from apar_workloads import build_trace, make_config, manual_tree, node_kv, step_q
    from oracle import DenseThreads

    w = make_config(w_name, seed=seed, n_requests=n_req)
    hd = w.heads
    n_thr = attended = 0
    t_dec = t_mat = 0.0
    with threadpool_limits(limits=1):
        for r in requests:
            idx = [n.idx for n in w.nodes if n.request == r]
            base = idx[0]
            sub = manual_tree([-1 if w.nodes[i].parent < 0 else w.nodes[i].parent - base for i in idx],
                              [w.nodes[i].seg_len for i in idx], hd, seed=seed + 1000 * r, data_scale=w.data_scale)
            dense = DenseThreads(hd.n_q_heads, hd.n_kv_heads, hd.head_dim)
            ops, live, _ = build_trace(sub)
            t0 = time.perf_counter()
            for op in ops:
                if op.kind == "create":
                    dense.create()
                elif op.kind == "append":
                    dense.append(op.tid, *node_kv(sub, op.node))
                elif op.kind == "fork":
                    dense.fork(op.tid, len(op.children))
                else:
                    dense.free(op.tid)
            q = step_q(sub, 0, len(live))
            t1 = time.perf_counter()
            dense.decode(q, live)
            t2 = time.perf_counter()
            t_mat += t1 - t0
            t_dec += t2 - t1
            n_thr += len(live)
            attended += sum(dense.length(t) for t in live)
    return os.getpid(), n_thr, attended, t_dec, t_mat


def cpu_baseline(w_name: str, seed: int, n_req: int, n_total: int):
    """The fp64 oracle, as it stands, on the first n_req requests of the same workload shapes, spread over
    the host cores with a process pool over requests (one BLAS thread per worker).  Runs before the GPU
    is touched, in spawned processes that import numpy and the oracle only; the rows are drawn on the host
    by the seeded recipe (their values do not change the oracle's work)."""
    import multiprocessing as mp

    from apar_workloads import make_config

    workers = max(1, min(16, os.cpu_count() or 1, n_req))  # a one-GPU machine gives a job 16 cores whatever it shows
    hd = make_config(w_name, seed=seed, n_requests=1).heads
    tasks = [(w_name, seed, n_req, list(range(i, n_req, 4 * workers))) for i in range(min(4 * workers, n_req))]
    t0 = time.perf_counter()
    with mp.get_context("spawn").Pool(workers) as pool:
        t_up = time.perf_counter() - t0
        t0 = time.perf_counter()
        got = list(pool.imap_unordered(_oracle_requests, tasks))
        wall = time.perf_counter() - t0
    per_pid = {}
    for pid, n, att, t_dec, t_mat in got:
        d = per_pid.setdefault(pid, [0.0, 0.0])
        d[0] += t_dec
        d[1] += t_mat
    n_thr = sum(g[1] for g in got)
    attended = sum(g[2] for g in got)
    dec = max(d[0] for d in per_pid.values())  # the decode phase ends when the slowest worker is done
    return {
        "value": n_thr / dec,
        "unit": "thread-queries/s",
        "cores": len(per_pid),
        "blas_threads_per_worker": 1,
        "host_cpus": os.cpu_count(),
        "kind": "oracle",
        "sample": f"first {n_req} of {n_total} requests of {w_name} (seed {seed}): {n_thr} threads, {attended} "
                  f"attended tokens, fp64 dense attention over deep-copied per-thread rows, a process pool over "
                  f"requests; decode time of the slowest of {len(per_pid)} workers {dec:.2f} s (sum over workers "
                  f"{sum(d[0] for d in per_pid.values()):.1f} s; materialising the copies another "
                  f"{sum(d[1] for d in per_pid.values()):.1f} s, not counted; whole pool.map {wall:.1f} s after "
                  f"{t_up:.1f} s of start-up)",
        "effective_GBps": attended * hd.kv_bytes_per_token / dec / 1e9,
    }


def read_traffic(workload: str, algorithmic_bytes: float):
    """HBM traffic of a launch as algorithmic bytes x (fetched + written) / algorithmic, the ratio taken from
    the committed rocprofv3 counter summary of the same workload (counters cannot be read from inside the
    run; the ratio, unlike the byte count, does not depend on how many steps a run takes).
    Returns (traffic bytes, ratio, source) or (None, None, None)."""
    path = os.path.join(ROOT, "profiles", f"attention_bf16_{workload}_pmc.txt")
    vals = {}
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 2 and not line.startswith("#"):
                try:
                    vals[f[0]] = float(f[1])
                except ValueError:
                    pass
    except OSError:
        return None, None, None
    need = ("fetch_bytes_per_launch", "write_bytes_per_launch", "algorithmic_bytes_per_launch_same_launches")
    if any(k not in vals for k in need):
        return None, None, None
    ratio = (vals[need[0]] + vals[need[1]]) / vals[need[2]]
    return algorithmic_bytes * ratio, ratio, os.path.relpath(path, ROOT)


def _pct(sorted_ms, p):
    return sorted_ms[min(len(sorted_ms) - 1, int(round(p * (len(sorted_ms) - 1))))] if sorted_ms else None


def spec_loop(args, w, K=None, warmup=None) -> dict:
    """The speculative decode loop: every step is multi-candidate attention (5 candidates per thread under
    a random tree mask), append of the accepted rows, release of finished threads, fork of new ones."""
    import torch

    import paper_2401_06761_amd as ap
    from paper_2401_06761_amd.driver import SpecRun

    hd = w.heads
    K = args.steps if K is None else K
    warmup = args.warmup if warmup is None else warmup
    t0 = time.perf_counter()
    run = SpecRun(w, K + warmup, n_cand=5, commit=not args.two_pass)
    t_dry = time.perf_counter() - t0
    run.build()
    if args.chunk:
        ap.apar_set_chunk_blocks(run.h, args.chunk)
    if args.no_plan_reuse:
        ap.apar_set_plan_reuse(run.h, False)
    if args.matrix_units:
        ap.apar_set_matrix_units(run.h, *(int(x) for x in args.matrix_units.split(",")))
    run.draw_ahead(warmup + K)  # the synthetic step plans (masks, accepted chains, coins) exist before the clock starts
    for _ in range(warmup):
        run.step()
    torch.cuda.synchronize()
    ap.apar_profile_read(run.h)
    ap.apar_profile_enable(run.h, True)
    n_q = alg = 0
    n0 = len(run.live)
    t0 = time.perf_counter()
    for _ in range(K):
        st = run.step()[0]
        info = ap.apar_last_plan_info(run.h)
        n_q += len(st.live)
        alg += info.algorithmic_bytes
    t_host = time.perf_counter() - t0
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = ap.apar_profile_read(run.h)
    calls_ms = sorted(ap.apar_profile_attention_calls(run.h))
    st1 = ap.apar_pool_stats(run.h)
    attn_ms = prof.attention_kernel_ms / K
    traffic, ratio, source = read_traffic("spec128", alg / K)
    result = {
        "metric": "decode-attn thread-queries/s + achieved HBM GB/s on fork-tree paged KV",
        "value": n_q / elapsed, "unit": "thread-queries/s", "n_gpus": 1, "steps": K, "warmup": warmup,
        "ms_per_step": elapsed / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": hd.dtype, "data": "synthetic",
        "config": {"workload": f"spec128: {w.n_requests} requests, depth-2 fork trees, then a {K}-step speculative "
                               f"loop with 5 candidates per thread (fork 0.02, finish 0.01 per step); "
                               f"{n0} -> {len(run.live)} live threads, seed {args.seed}",
                   "accepted_rows": "gathered and appended in a second pass" if args.two_pass
                   else "committed straight from the candidate arrays"},
        "candidate_queries_per_s": 5 * n_q / elapsed,
        "roofline": {"bound": "hbm", "kernel": "attention_bf16 (multi-candidate call)",
                     "achieved": (alg / K) / (attn_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": (alg / K) / (attn_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_over_algorithmic": ratio, "traffic_ratio_from": source,
                     "algorithmic_bytes_per_launch": alg / K, "kernel_ms_per_launch": attn_ms,
                     "kernel_ms_median_p10_p90": [_pct(calls_ms, 0.5), _pct(calls_ms, 0.1), _pct(calls_ms, 0.9)]},
        "breakdown_ms_per_step": {"attention_kernel": attn_ms, "merge_kernel": prof.merge_kernel_ms / K,
                                  "append_kernels": prof.append_kernels_ms / K, "plan_host": prof.plan_host_ms / K,
                                  "host_issue": t_host / K * 1e3, "host_waiting_for_gpu": prof.host_wait_ms / K},
        "host_share_of_wall": (t_host - prof.host_wait_ms * 1e-3) / elapsed,
        "peak_blocks": run.peak_blocks, "peak_threads": run.peak_threads, "dry_run_s": t_dry,
        "kv_bytes": {"resident": st1.bytes_resident, "vanilla_copy_each_prefix": st1.bytes_vanilla,
                     "ratio": st1.bytes_vanilla / max(st1.bytes_resident, 1)},
    }
    run.close()
    return result


def prefill_bench(args, w) -> int:
    """Secondary measurement: tree-masked prefill attention (apar_prefill_attention) over the segments of a
    resident fork-tree workload.  MFMA-bound, so the roofline is the dense bf16 matrix-core peak."""
    import numpy as np
    import torch

    import paper_2401_06761_amd as ap
    from apar_workloads import rows_device
    from paper_2401_06761_amd.driver import TreeRun

    hd = w.heads
    run = TreeRun(w, headroom_steps=8, device="cuda:0")
    run.build()
    ap.apar_set_prefill_kernel(run.h, {"auto": ap.APAR_PREFILL_AUTO, "row_tiles": ap.APAR_PREFILL_ROW_TILES,
                                       "matrix": ap.APAR_PREFILL_MATRIX}[args.prefill_kernel])
    kernel_names = {ap.APAR_PREFILL_ROW_TILES: "attention_bf16 (prefill plan)", ap.APAR_PREFILL_MATRIX: "prefill_bf16"}
    live = np.asarray(run.live, dtype=np.int32)
    lens = np.array([ap.apar_thread_len(run.h, int(t)) for t in live], dtype=np.int64)
    own = np.array([w.nodes[run.node_of[int(t)]].seg_len for t in live], dtype=np.int64)
    results = {}
    for name, m in (("own_segments", own), ("whole_paths", lens)):
        if name == "whole_paths" and int(m.sum()) > 4_000_000:
            continue  # (the q and out rows alone would take tens of GB)
        rows = int(m.sum())
        q = rows_device(w, 21, 0, (rows, hd.n_q_heads, hd.head_dim), "cuda:0")
        out = torch.empty_like(q)
        m32 = m.astype(np.int32)
        for _ in range(args.warmup):
            ap.apar_prefill_attention(run.h, q, live, m32, out)
        torch.cuda.synchronize()
        ap.apar_profile_read(run.h)
        ap.apar_profile_enable(run.h, True)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            ap.apar_prefill_attention(run.h, q, live, m32, out)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        prof = ap.apar_profile_read(run.h)
        ap.apar_profile_enable(run.h, False)
        info = ap.apar_last_plan_info(run.h)
        flops = 4.0 * hd.head_dim * hd.n_q_heads * info.path_tokens
        ms = prof.attention_kernel_ms / args.steps
        results[name] = {"query_tokens": rows, "attended_pairs": int(info.path_tokens), "flop_per_call": flops,
                         "kernel_ms_per_call": ms, "wall_ms_per_call": wall / args.steps * 1e3,
                         "plan_host_ms_per_call": prof.plan_host_ms / args.steps,
                         "tflops": flops / (ms * 1e-3) / 1e12, "workgroups": int(info.n_units),
                         "kernel": kernel_names[ap.apar_last_prefill_kernel(run.h)]}
        del q, out
    main_r = results["own_segments"]
    line = {
        "metric": "tree-masked prefill attention, query tokens/s (secondary; the headline is the decode step)",
        "value": main_r["query_tokens"] / (main_r["wall_ms_per_call"] * 1e-3), "unit": "query-tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_r["wall_ms_per_call"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": hd.dtype, "data": "synthetic",
        "config": {"workload": f"{args.config} forest resident in the pool ({len(live)} live threads); one call = "
                               f"prefill attention of every live thread's own segment under the tree mask"},
        "roofline": {"bound": "mfma", "kernel": main_r["kernel"], "achieved": main_r["tflops"],
                     "peak": 2500.0, "unit": "TFLOP/s", "frac": main_r["tflops"] / 2500.0, "traffic": None},
        "cases": results,
    }
    run.close()
    print(json.dumps(line))
    return 0


def shared_prefix_bench(args) -> int:
    """Secondary measurement: decode attention when several hundred query rows share one long prefix
    (16 requests, a root of `root` tokens forked into 512 one-token leaves, 32 MHA heads): the root is more
    rows than a fused workgroup carries: it is inlined (read again by every unit of 128 rows below it, nothing
    to merge) or stands alone with partial results, on the row-tile kernel or on the 32x32 matrix-core kernel
    (the default from 2048 tokens on).  Times the variants for two root lengths."""
    import numpy as np
    import torch

    import paper_2401_06761_amd as ap
    from apar_workloads import HeadConfig, manual_tree
    from paper_2401_06761_amd.driver import TreeRun

    n_req, fan = 16, 512
    cases = {}
    for root in (4096, 1024):
        parents, segs = [], []
        for _ in range(n_req):
            base = len(parents)
            parents.append(-1)
            segs.append(root)
            parents += [base] * fan
            segs += [1] * fan
        w = manual_tree(parents, segs, HeadConfig(32, 32, 128, "bf16"), seed=args.seed, data_scale=0.09)
        run = TreeRun(w, headroom_steps=4, churn=0.0)
        run.build()
        ids = np.asarray(run.live, dtype=np.int32)
        q, out = run.banks[0][0], run.out
        res = {}
        for name, inline, knob in (("inlined", True, (0, 1)), ("stand_alone_row_tile_units", False, (0, 1)),
                                   ("stand_alone_matrix_units", False, (1, 1)), ("default", True, (256, 128))):
            ap.apar_set_inline_shared(run.h, inline)
            ap.apar_set_matrix_units(run.h, *knob)
            for _ in range(args.warmup):
                ap.apar_decode_attention(run.h, q, ids, out)
            torch.cuda.synchronize()
            ap.apar_profile_read(run.h)
            ap.apar_profile_enable(run.h, True)
            for _ in range(args.steps):
                ap.apar_decode_attention(run.h, q, ids, out)
            torch.cuda.synchronize()
            prof = ap.apar_profile_read(run.h)
            ap.apar_profile_enable(run.h, False)
            info = ap.apar_last_plan_info(run.h)
            ms = prof.attention_kernel_ms / args.steps
            res[name] = {"attention_kernel_ms": ms, "merge_kernel_ms": prof.merge_kernel_ms / args.steps,
                         "tflops": 4.0 * 128 * 32 * info.path_tokens / (ms * 1e-3) / 1e12,
                         "achieved_gb_s": info.algorithmic_bytes / (ms * 1e-3) / 1e9}
        cases[f"root_{root}"] = res
        run.close()
    main_r = cases["root_4096"]["default"]
    print(json.dumps({
        "metric": "decode attention over a prefix shared by 512 threads (secondary; the headline is the ht256 decode step)",
        "value": n_req * fan / (main_r["attention_kernel_ms"] * 1e-3), "unit": "thread-queries/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_r["attention_kernel_ms"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{n_req} requests, root of 4096 tokens forked into {fan} one-token leaves, Hq=Hkv=32, d=128"},
        "roofline": {"bound": "mfma", "kernel": "attention_units_bf16 + attention_bf16", "achieved": main_r["tflops"],
                     "peak": 2500.0, "unit": "TFLOP/s", "frac": main_r["tflops"] / 2500.0, "traffic": None},
        "cases": cases}))
    return 0


def serving_bench(args) -> int:
    """Secondary measurement: throughput of the serving loop against the size of the KV pool, for APAR
    decoding and for the sequential stand-in of the same responses (the shape of the paper's
    throughput-vs-cache-memory experiment, Sec. 3.3), on synthetic requests."""
    import numpy as np
    import torch

    import paper_2401_06761_amd as ap
    from apar_workloads import SamplerConfig, make_requests
    from paper_2401_06761_amd.serving import ServingRun

    n_q = n_kv = 32
    d = 128
    cfg = SamplerConfig()
    reqs = make_requests(args.requests or 256, seed=args.seed)
    cap = args.max_running
    # responses and the cache a sequential decoder needs for them at this concurrency: dry runs
    dry = ap.Pool(n_q, n_kv, d, "bf16", 1 << 22, max_threads=1 << 30, dry_run=True)
    a = ServingRun(dry, reqs, cfg, cap, 0)
    sa = a.run()
    a.close()
    flat = {r.rid: r.prompt_len + len(a.outputs[r.rid]) for r in reqs}
    b = ServingRun(dry, reqs, cfg, cap, 0, flat_lengths=flat)
    sb = b.run()
    b.close()
    dry.close()
    full = int(sb["peak_used_blocks"])
    longest = max(flat.values())
    dev = "cuda:0"
    gen = torch.Generator(device=dev).manual_seed(args.seed)
    qb = (0.09 * torch.randn((4096, n_q, d), generator=gen, device=dev)).to(torch.bfloat16)
    kb = (0.09 * torch.randn((8192, n_kv, d), generator=gen, device=dev)).to(torch.bfloat16)
    vb = (0.09 * torch.randn((8192, n_kv, d), generator=gen, device=dev)).to(torch.bfloat16)
    rows = []
    for frac in (0.1, 0.2, 0.4, 0.8, 1.0):
        n_blocks = max(int(frac * full), (longest + 15) // 16 * 2 + 8)
        for mode in ("apar", "sequential"):
            pool = ap.Pool(n_q, n_kv, d, "bf16", n_blocks, max_threads=1 << 24, device=dev)
            run = ServingRun(pool, reqs, cfg, cap, max(1, n_blocks // 100),
                             flat_lengths=None if mode == "apar" else flat, banks=(qb, kb, vb))
            st = run.run()
            assert st["finished"] == len(reqs)
            st.update({"mode": mode, "pool_fraction": frac, "pool_blocks": n_blocks,
                       "pool_GB": n_blocks * ap.apar_pool_stats(pool.handle).block_bytes / 1e9,
                       "output_tokens_per_s": st["useful_tokens"] / st["wall_s"],
                       "ms_per_step": st["wall_s"] / max(st["steps"], 1) * 1e3})
            rows.append(st)
            run.close()
            pool.close()
    best = max(r["output_tokens_per_s"] for r in rows if r["mode"] == "apar")
    line = {
        "metric": "serving loop output tokens/s against KV pool size (secondary; the headline is the decode step)",
        "value": best, "unit": "output-tokens/s", "n_gpus": 1, "steps": int(sa["steps"]), "warmup": 0,
        "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{len(reqs)} synthetic requests queued at the start (prompts 16..256 tokens, up to "
                               f"{cfg.max_threads} threads per response, fork {cfg.p_fork} / eos {cfg.p_eos} per token), "
                               f"at most {cap} running, Hq=Hkv=32 d=128; pool sized as a fraction of the "
                               f"{full} blocks the sequential decoder peaks at"},
        "sweep": rows,
    }
    print(json.dumps(line))
    return 0


def tree_bench(args, name: str, steps: int, warmup: int, n_requests=None, kv_fp8: bool = False) -> dict:
    """Decode steps over one resident fork-tree workload (mha64, ht256, gqa1024); returns the result line.
    kv_fp8: the same workload on a pool that keeps full blocks in fp8 (bf16 at the interface)."""
    import torch

    import paper_2401_06761_amd as ap
    from apar_workloads import make_config
    from paper_2401_06761_amd.driver import TreeRun

    dev = "cuda:0"
    w = make_config(name, seed=args.seed, n_requests=n_requests, kv_fp8=kv_fp8)
    hd = w.heads
    t_build = time.perf_counter()
    run = TreeRun(w, headroom_steps=steps + warmup + 8, churn=args.churn, device=dev)
    run.build()
    t_build = time.perf_counter() - t_build
    if args.chunk:
        ap.apar_set_chunk_blocks(run.h, args.chunk)
    if args.no_plan_reuse:
        ap.apar_set_plan_reuse(run.h, False)
    if args.matrix_units:
        ap.apar_set_matrix_units(run.h, *(int(x) for x in args.matrix_units.split(",")))
    st0 = ap.apar_pool_stats(run.h)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(warmup):
        run.step()
    torch.cuda.synchronize()
    ap.apar_profile_read(run.h)
    ap.apar_profile_enable(run.h, True)
    plans0 = ap.apar_plan_counts(run.h)
    alg_bytes = 0
    unique_tokens = path_tokens = 0
    n_queries = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run.step()
        info = ap.apar_last_plan_info(run.h)
        alg_bytes += info.algorithmic_bytes
        unique_tokens += info.unique_tokens
        path_tokens += info.path_tokens
        n_queries += info.n_threads
    t_host = time.perf_counter() - t0
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = ap.apar_profile_read(run.h)
    calls_ms = sorted(ap.apar_profile_attention_calls(run.h))
    ap.apar_profile_enable(run.h, False)
    st1 = ap.apar_pool_stats(run.h)
    info = ap.apar_last_plan_info(run.h)
    plans = [a - b for a, b in zip(ap.apar_plan_counts(run.h), plans0)]

    K = steps
    attn_ms = prof.attention_kernel_ms / K
    merge_ms = prof.merge_kernel_ms / K
    append_ms = prof.append_kernels_ms / max(prof.n_append_calls, 1)
    achieved = (alg_bytes / K) / (attn_ms * 1e-3) / 1e9
    traffic, ratio, source = read_traffic(w.name, alg_bytes / K)
    result = {
        "metric": "decode-attn thread-queries/s + achieved HBM GB/s on fork-tree paged KV",
        "value": n_queries / elapsed,
        "unit": "thread-queries/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": warmup,
        "ms_per_step": elapsed / K * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if kv_fp8 else hd.dtype,
        "data": "synthetic",
        "config": {
            "kv_cache": "full blocks in fp8 (e4m3, one power-of-two scale per block, kv head and K|V), filling "
                        "blocks bf16; matrix-core arithmetic in bf16" if kv_fp8 else hd.dtype,
            "workload": f"{name}: {w.n_requests} requests, fork trees of depth "
                        f"{max(n.depth for n in w.nodes)}, {len(run.live)} live threads, Hq={hd.n_q_heads} "
                        f"Hkv={hd.n_kv_heads} d={hd.head_dim} block=16, seed {args.seed}",
            "step": "fork+free churn %.3g of threads, append 1 KV row per thread, decode attention over all "
                    "threads" % args.churn,
            "threads_per_step": n_queries // K,
            "unique_kv_tokens_per_step": unique_tokens // K,
            "attended_tokens_per_step": path_tokens // K,
        },
        "roofline": {
            "bound": "hbm",
            "kernel": "attention_bf16 (fp8 tiles)" if kv_fp8 else "attention_bf16",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": traffic,
            "traffic_over_algorithmic": ratio,
            "traffic_ratio_from": source,
            "algorithmic_bytes_per_launch": alg_bytes / K,
            "kernel_ms_per_launch": attn_ms,
            "kernel_ms_median_p10_p90": [_pct(calls_ms, 0.5), _pct(calls_ms, 0.1), _pct(calls_ms, 0.9)],
        },
        "breakdown_ms_per_step": {
            "attention_kernel": attn_ms,
            "merge_kernel": merge_ms,
            "append_kernels": append_ms,
            "plan_host": prof.plan_host_ms / K,
            "host_issue": t_host / K * 1e3,
            "host_waiting_for_gpu": prof.host_wait_ms / K,
        },
        "attention_call_thread_queries_per_s": (n_queries / K) / ((attn_ms + merge_ms) * 1e-3),
        "attention_call_end_to_end_thread_queries_per_s":  # plan building on the host counted serially
            (n_queries / K) / ((attn_ms + merge_ms + prof.plan_host_ms / K) * 1e-3),
        "kv_bytes": {
            "resident": st1.bytes_resident,
            "vanilla_copy_each_prefix": st1.bytes_vanilla,
            "ratio": st1.bytes_vanilla / max(st1.bytes_resident, 1),
            "resident_after_build": st0.bytes_resident,
            "vanilla_after_build": st0.bytes_vanilla,
        },
        "plan": {"segments": info.n_segments, "units": info.n_units, "partial_rows": info.n_partial_rows,
                 "unique_blocks": info.unique_blocks,
                 "calls_that_built_it": plans[0], "calls_that_carried_the_previous_one_over": plans[1]},
        "build_s": t_build,
    }
    run.close()
    del run
    torch.cuda.empty_cache()
    return result


def _secondary_view(r: dict) -> dict:
    """What the headline line keeps of another configuration's result."""
    keep = ("value", "unit", "steps", "warmup", "ms_per_step", "config", "roofline", "breakdown_ms_per_step",
            "kv_bytes", "candidate_queries_per_s", "attention_call_thread_queries_per_s", "build_s")
    return {k: r[k] for k in keep if k in r}


def main() -> int:
    ap_ = argparse.ArgumentParser()
    ap_.add_argument("--gpus", type=int, default=1)
    ap_.add_argument("--steps", type=int, default=50)
    ap_.add_argument("--warmup", type=int, default=10)
    ap_.add_argument("--config", default="ht256", choices=["mha64", "ht256", "gqa1024", "spec128"])
    ap_.add_argument("--seed", type=int, default=0)
    ap_.add_argument("--requests", type=int, default=None, help="first n requests only (debugging)")
    ap_.add_argument("--chunk", type=int, default=None, help="blocks per work unit")
    ap_.add_argument("--churn", type=float, default=0.01)
    ap_.add_argument("--no-plan-reuse", action="store_true",
                     help="build every decode call's plan afresh instead of carrying the previous call's over")
    ap_.add_argument("--cpu-requests", type=int, default=128,
                     help="requests of the workload the oracle decodes for the cpu_baseline leg")
    ap_.add_argument("--no-cpu-baseline", action="store_true",
                     help="skip the oracle (use under rocprofv3: the leg starts worker processes)")
    ap_.add_argument("--no-secondary", action="store_true",
                     help="only the named configuration (default: ht256 as the headline plus mha64, gqa1024 and a "
                          "spec128 loop under 'secondary')")
    ap_.add_argument("--spec-steps", type=int, default=256, help="steps of the secondary spec128 loop")
    ap_.add_argument("--prefill-kernel", choices=("auto", "row_tiles", "matrix"), default="auto",
                     help="with --prefill: let the library choose the kernel per call, or force one")
    ap_.add_argument("--matrix-units", default=None, metavar="ROWS,BLOCKS",
                     help="thresholds from which a stand-alone shared segment runs on the 32x32 kernel (library default 256,128; 0,0 never)")
    ap_.add_argument("--shared-prefix", action="store_true",
                     help="measure decode attention over long prefixes shared by 512 threads, row-tile vs matrix units")
    ap_.add_argument("--prefill", action="store_true",
                     help="measure apar_prefill_attention over the workload's segments instead of the decode step")
    ap_.add_argument("--serving", action="store_true",
                     help="measure the serving loop (admission, early release, preemption) against the pool size")
    ap_.add_argument("--max-running", type=int, default=64)
    ap_.add_argument("--two-pass", action="store_true",
                     help="spec128: gather the accepted rows on the caller's side and append them with "
                          "apar_append_kv_batch instead of apar_commit_candidates")
    ap_.add_argument("--kv-fp8", action="store_true",
                     help="mha64 / ht256 / gqa1024 on a pool that keeps full KV blocks in fp8 (half the bytes per cached token)")
    ap_.add_argument("--copy-calibration", action="store_true",
                     help="also run one plain 4 GiB device copy (reference for HBM byte counters)")
    args = ap_.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path would shard by request, each GPU with a pool of "
              "its own and nothing to exchange); --gpus must be 1", file=sys.stderr)
        return 2
    special = args.shared_prefix or args.serving or args.prefill
    headline_default = not special and args.config == "ht256" and args.requests is None and not args.kv_fp8

    # The oracle leg comes first: it starts worker processes, which must happen before this process touches the GPU.
    cpu = None
    if not special and not args.no_cpu_baseline:
        from apar_workloads import make_config as _mk

        n_total = _mk(args.config, seed=args.seed, n_requests=args.requests).n_requests
        cpu = cpu_baseline(args.config, args.seed, min(args.cpu_requests, n_total), n_total)

    import torch

    from apar_workloads import make_config

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    if args.shared_prefix:
        return shared_prefix_bench(args)
    if args.serving:
        return serving_bench(args)
    w = make_config(args.config, seed=args.seed, n_requests=args.requests)
    if args.prefill:
        return prefill_bench(args, w)
    if args.config == "spec128":
        result = spec_loop(args, w)
    else:
        result = tree_bench(args, args.config, args.steps, args.warmup, args.requests, kv_fp8=args.kv_fp8)
    if cpu is not None:
        result["cpu_baseline"] = cpu
    if headline_default and not args.no_secondary:
        # the other configurations, each a run of its own after the headline's pool is gone; short enough
        # for the whole command to stay within a couple of minutes
        sec = {}
        sec["mha64"] = _secondary_view(tree_bench(args, "mha64", min(args.steps, 50), min(args.warmup, 10)))
        sec["gqa1024"] = _secondary_view(tree_bench(args, "gqa1024", min(args.steps, 20), min(args.warmup, 5)))
        sec["spec128_loop"] = _secondary_view(spec_loop(args, make_config("spec128", seed=args.seed),
                                                        K=args.spec_steps, warmup=0))
        sec["ht256_fp8_kv_cache"] = _secondary_view(tree_bench(args, "ht256", args.steps, args.warmup, kv_fp8=True))
        result["secondary"] = sec
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
