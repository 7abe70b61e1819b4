#!/usr/bin/env python3
"""Benchmark of the MixKV compression step on one MI355X.

One step = one mixkv_compress call over a whole synthetic cache (all layers, all KV heads):
score -> mix -> top-B -> gather.  Default workload: the Qwen2-VL-7B-shaped 28-layer, 8K-token
cache (workload "c3"), budget 64.  Prints ONE JSON line.

  ms_per_step  median of the timed steps, each bracketed by HIP events on the launch stream (the
               wall-clock mean over the same steps is reported beside it); inputs resident in HBM,
               three copies of the cache used round-robin so that every step streams from HBM
  value        cached tokens compressed per second: batch * N / ms_per_step
  other_budgets_and_warm   the same figure at budgets 128 / 256 / 512 and, for the default budget, on
               a single copy of the cache (default workload only)
  roofline     the dominant kernel's algorithmic bytes per launch / its median duration, measured
               with HIP events on the launch stream (mixkv_compress_profiled), against 8 TB/s
  cpu_baseline the float64 oracle on the same inputs on the host cores (process pool), before the
               GPU is touched
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

os.environ.setdefault("OMP_NUM_THREADS", "1")      # one BLAS thread per oracle worker

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2510_20707_amd import synth  # noqa: E402

HBM_PEAK = 8.0e12
MFMA_BF16_PEAK = 2.5e15
# HBM bytes per launch (fetched + written) of the two streaming kernels on the default workload, from
# rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this command scaled by a 1 GiB copy kernel (summary and
# commands: profiles/mixkv_compress_c3_b64_hbm_traffic.md).  A profile describes the kernels it was
# taken on: the record carries a hash of their sources, and the bench line reports the figure only for
# the profiled command (default workload, budget and variant, three copies) and unchanged sources.
PROFILED_TRAFFIC = {
    "sources": ["mixkv_stream.hip", "mixkv_stream.h"],
    "sources_sha256": "f75b42fdd250bd95552541286be4fc687cbc665876eb759294aec97b0497374a",
    "kernels": {"stats": ("stats_kernel<bf16,128,8,1>", 513.6e6), "attn": ("attn_kernel<bf16,128,4,2,spare>", 278.3e6)},
}


def kernel_sources_sha256(names):
    import hashlib
    h = hashlib.sha256()
    for n in names:
        with open(os.path.join(ROOT, "paper_2510_20707_amd", "csrc", n), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def profiled_traffic(args, wl, stage):
    """The profiled HBM bytes per launch of `stage`'s kernel, or None if this run is not the profiled one."""
    default = (args.workload == "c3" and wl.n_layers == 28 and args.budget in (None, 64) and args.copies == 3
               and args.intrinsic == "vnorm" and args.mix == "head_adaptive" and not args.given_lse
               and args.budgets == "config")
    if not default or stage not in PROFILED_TRAFFIC["kernels"]:
        return None
    if kernel_sources_sha256(PROFILED_TRAFFIC["sources"]) != PROFILED_TRAFFIC["sources_sha256"]:
        return None
    name, nbytes = PROFILED_TRAFFIC["kernels"][stage]
    return {"kernel": name, "bytes_per_launch": nbytes, "profile": "profiles/mixkv_compress_c3_b64_hbm_traffic.md"}


def timed_steps(calls, steps, warmup, stream):
    """`warmup` untimed steps, then `steps` steps each bracketed by HIP events on the launch stream
    (no host synchronisation in between).  Returns (wall-clock mean, per-step event times), in ms."""
    import torch
    for i in range(warmup):
        calls[i % len(calls)].compress(stream)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evs[0].record(stream)
    for i in range(steps):
        calls[i % len(calls)].compress(stream)
        evs[i + 1].record(stream)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps * 1e3
    return wall, [evs[i].elapsed_time(evs[i + 1]) for i in range(steps)]


_LAYERS = None
_WL = None
_BUDGET = None
_VARIANT = ("vnorm", "head_adaptive")
_RGIVEN = None
_HEAD_BUDGETS = None
_LSE = None


def _oracle_layer(l):
    from oracle import mixkv_oracle as O
    wl = _WL
    hb = _HEAD_BUDGETS
    p = O.Params(wl.n_q_heads, wl.n_kv_heads, wl.window, _BUDGET, pool=wl.pool, pool_kernel=wl.pool_kernel,
                 softmax_scale=wl.softmax_scale, eps=wl.eps, budget_mode=wl.budget_mode if hb is None else "per_head",
                 budget_floor=wl.budget_floor, intrinsic=_VARIANT[0], mix=_VARIANT[1])
    out = O.compress_layer(_LAYERS[l].K, _LAYERS[l].V, _LAYERS[l].Q, p, None if _RGIVEN is None else _RGIVEN[l],
                           None if hb is None else hb[l], None if _LSE is None else _LSE[l].astype(np.float64))
    return l, [[i.astype(np.int32) for i in row] for row in out["indices"]], out["scores"].astype(np.float32)


def cpu_baseline(wl, layers, budget, max_layers, variant, r_given, head_budgets, lse):
    """Time the oracle as it stands on a bounded sample (the first `max_layers` layers)."""
    import multiprocessing as mp
    global _LAYERS, _WL, _BUDGET, _VARIANT, _RGIVEN, _HEAD_BUDGETS, _LSE
    _LAYERS, _WL, _BUDGET, _VARIANT, _RGIVEN, _HEAD_BUDGETS, _LSE = layers, wl, budget, variant, r_given, head_budgets, lse
    n = min(max_layers, len(layers))
    workers = max(1, min(n, len(os.sched_getaffinity(0)), int(os.environ.get("MIXKV_BENCH_WORKERS", "16"))))
    ctx = mp.get_context("fork")                   # children inherit the generated layers; no GPU state exists yet
    with ctx.Pool(workers) as pool:
        pool.map(abs, range(workers))              # spin the workers up outside the timed region
        t0 = time.perf_counter()
        res = pool.map(_oracle_layer, range(n), chunksize=1)
        dt = time.perf_counter() - t0
    # scaled to the metric: tokens of the whole cache per second if every layer cost what the sample did
    tokens_per_s = wl.batch * wl.seq_len / (dt * len(layers) / n)
    cpu_model = "unknown CPU"
    try:
        with open("/proc/cpuinfo") as f:
            cpu_model = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), cpu_model)
    except OSError:
        pass
    return dict(value=tokens_per_s, unit="tokens/s", cores=workers, kind="oracle",
                sample=f"{n} of {len(layers)} layers ({n * wl.batch * wl.n_kv_heads} units) in {dt:.2f} s, "
                       f"process pool of {workers} on {cpu_model}, 1 BLAS thread each; scaled by {len(layers)}/{n}"), \
        {r[0]: r for r in res}


def algorithmic_bytes(wl, budget, scores_out, reads_v=True):
    """Bytes the method itself must move per unit: K once, V once (only when the value norm is
    scored), the window queries, the kept rows read and written, the indices; optionally the N-long
    score vector."""
    e = 2 if wl.dtype == "bf16" else 4
    n, d = wl.seq_len, wl.head_dim
    per_unit = n * d * e * (2 if reads_v else 1) + wl.group * wl.window * d * e + 4 * budget * d * e + 4 * budget
    if scores_out:
        per_unit += 4 * n
    return per_unit


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3", choices=sorted(synth.WORKLOADS))
    ap.add_argument("--budget", type=int, default=None)
    ap.add_argument("--layers", type=int, default=None, help="use only the first L layers (not the headline)")
    ap.add_argument("--copies", type=int, default=3, help="distinct device copies of the cache, used round-robin")
    ap.add_argument("--cpu-layers", type=int, default=28, help="layers the oracle baseline runs (0 = skip)")
    ap.add_argument("--no-parity", action="store_true")
    ap.add_argument("--no-sweep", action="store_true",
                    help="skip the extra figures of the default workload (budgets 128 / 256 / 512 and the warm run)")
    ap.add_argument("--intrinsic", default="vnorm", choices=["none", "vnorm", "knorm"],
                    help="intrinsic importance; anything but vnorm is an ablation variant, not the headline")
    ap.add_argument("--mix", default="head_adaptive", choices=["head_adaptive", "sum", "div_only", "imp_only", "given_r"],
                    help="score mix; anything but head_adaptive is an ablation variant, not the headline")
    ap.add_argument("--calibrate-copy-mib", type=int, default=0,
                    help="also launch an elementwise copy kernel that reads and writes this many MiB: a kernel of "
                         "known traffic against which rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled")
    ap.add_argument("--given-lse", action="store_true",
                    help="hand the window rows' log-sum-exp to the library, as a prefill attention kernel would "
                         "(the first pass then computes no logits); a variant, not the headline")
    ap.add_argument("--decode-tail", type=int, default=-1,
                    help="also time mixkv_decode_attention (one new token per layer over the cache just compacted "
                         "plus this many appended rows); reported in an extra 'decode' object")
    ap.add_argument("--similarity-block", type=int, default=0,
                    help="also time mixkv_similarity (redundancy analysis of the keys: r and the heat-map at this "
                         "block size) on the same cache; reported in an extra 'similarity' object")
    ap.add_argument("--budgets", default="config", choices=["config", "pyramid"],
                    help="pyramid: budgets given per layer, falling linearly from 2B-W in the first layer to W in the "
                         "last (mean B); a per-head-table variant of a fixed-budget workload, not the headline")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no cross-GPU step); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    wl = synth.WORKLOADS[args.workload]
    if args.layers:
        wl = wl.with_(n_layers=args.layers)
    budget = args.budget or wl.budget
    t0 = time.perf_counter()
    layers = [synth.make_layer(wl, l) for l in range(wl.n_layers)]
    t_gen = time.perf_counter() - t0

    r_given = None
    if args.mix == "given_r":       # seeded stand-in for head weights measured offline
        r_given = [np.random.default_rng([977, wl.cfg_id, l]).uniform(0, 1, (wl.batch, wl.n_kv_heads)).astype(np.float32)
                   for l in range(wl.n_layers)]
    head_budgets = None
    if args.budgets == "pyramid":
        if wl.budget_mode != "fixed":
            sys.exit("bench.py: --budgets pyramid needs a fixed-budget workload")
        per_layer = np.round(np.linspace(2 * budget - wl.window, wl.window, wl.n_layers)).astype(np.int32)
        head_budgets = np.repeat(per_layer[:, None], wl.n_kv_heads, axis=1)
    budget_mode = wl.budget_mode if head_budgets is None else "per_head"
    capacity = budget if head_budgets is None else int(head_budgets.max())      # rows per head in the output buffers
    lse = [synth.window_lse(wl, lay) for lay in layers] if args.given_lse else None
    cpu, oracle_res = (None, {})
    if args.cpu_layers > 0:
        cpu, oracle_res = cpu_baseline(wl, layers, budget, args.cpu_layers, (args.intrinsic, args.mix), r_given,
                                       head_budgets, lse)

    import torch
    from paper_2510_20707_amd import binding as B
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    p = B.make_params(wl.dtype, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.seq_len, wl.window, capacity,
                      pool=wl.pool, pool_kernel=wl.pool_kernel, softmax_scale=wl.softmax_scale, eps=wl.eps,
                      budget_mode=budget_mode, budget_floor=wl.budget_floor, intrinsic=args.intrinsic, mix=args.mix,
                      head_budgets=head_budgets)

    def up(a):
        if wl.dtype == "bf16":
            return torch.from_numpy(synth.round_to_bf16_bits(a).view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    base = [(up(l.K), up(l.V), up(l.Q)) for l in layers]
    copies = [base] + [[(k.clone(), v.clone(), q.clone()) for k, v, q in base] for _ in range(max(0, args.copies - 1))]
    # the importance-only score reads no key statistics: without a redundancy output the library skips them
    want_r = not (args.mix == "imp_only" and args.intrinsic != "knorm")
    outs = [B.alloc_layer_out(p, dev, scores=False, redundancy=want_r) for _ in layers]
    ws = B.alloc_workspace(p, len(layers), dev)
    rg_dev = None if r_given is None else [torch.from_numpy(r).to(dev) for r in r_given]
    lse_dev = None if lse is None else [torch.from_numpy(x).to(dev) for x in lse]
    calls = [B.PreparedCall(p, [x[0] for x in c], [x[1] for x in c], [x[2] for x in c], outs, ws, rg_dev, lse_dev)
             for c in copies]
    stream = torch.cuda.current_stream()

    if args.calibrate_copy_mib > 0:
        src = torch.ones(args.calibrate_copy_mib * (1 << 18), dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)           # one vectorised elementwise kernel: reads and writes the size once
        torch.cuda.synchronize()
        del src, dst

    wall_ms, per_step = timed_steps(calls, args.steps, args.warmup, stream)
    ms_per_step = float(np.median(per_step))          # the headline: median of the event-timed steps
    dt = ms_per_step * 1e-3 * args.steps                # (kept in seconds for the rates below)

    # per-kernel durations with HIP events on the launch stream, same inputs, same round-robin
    stage_runs = {}
    nprof = max(3, min(args.steps, 20))
    for i in range(nprof):
        for k, v in calls[i % len(calls)].compress_profiled(stream).items():
            stage_runs.setdefault(k, []).append(v)
    stage_ms = {k: float(np.median(v)) for k, v in stage_runs.items()}      # median over the profiled calls

    parity = None
    if oracle_res and not args.no_parity:
        # the last profiled call ran on copy (nprof-1) % copies; all copies hold the same values
        torch.cuda.synchronize()
        same, total = 0, 0
        for l, (_, idx_o, _) in oracle_res.items():
            idx_g = outs[l].indices.cpu().numpy()
            for b in range(wl.batch):
                off = 0
                for h in range(wl.n_kv_heads):
                    n = idx_o[b][h].shape[0]
                    g = idx_g[b, h] if budget_mode == "fixed" else idx_g.reshape(wl.batch, -1)[b, off:off + n]
                    same += int(np.array_equal(g, idx_o[b][h]))
                    total += 1
                    off += n
        parity = dict(units=total, identical_index_sets=same,
                      note="sets may differ only by near-ties inside the 2e-3 band; tests/ apply the band rule")

    units = wl.n_units
    e = 2 if wl.dtype == "bf16" else 4
    dec = None
    if args.decode_tail >= 0:
        t = args.decode_tail
        gen = torch.Generator(device=dev).manual_seed(7)
        dt_ = B.TORCH_DTYPE[p.dtype]
        qn = [(torch.randn((wl.batch, wl.n_q_heads, wl.head_dim), generator=gen, device=dev) * 0.3).to(dt_) for _ in layers]
        tails = [(torch.randn((wl.batch, wl.n_kv_heads, max(t, 1), wl.head_dim), generator=gen, device=dev).to(dt_),
                  torch.randn((wl.batch, wl.n_kv_heads, max(t, 1), wl.head_dim), generator=gen, device=dev).to(dt_))
                 for _ in layers]
        dout = [torch.empty_like(q) for q in qn]
        rows = units * (budget + t)                                              # rows read, K and V each
        dec_bytes = rows * wl.head_dim * e * 2 + 2 * len(layers) * wl.batch * wl.n_q_heads * wl.head_dim * e
        # Copies of the compacted cache, used round-robin, so that a call finds as little of its rows in the
        # chip's caches as a decoding step would (the model's weights stream through between two steps): as
        # many as it takes to pass twice the 256 MB Infinity Cache, at most eight.
        import types
        ncop = max(1, min(8, -(-2 * 256 * 2 ** 20 // dec_bytes)))
        dcalls = [B.PreparedDecode(p, outs, tails, qn, dout, t)]
        for _ in range(ncop - 1):
            clone = [types.SimpleNamespace(K_out=o.K_out.clone(), V_out=o.V_out.clone(), counts=o.counts, offsets=o.offsets)
                     for o in outs]
            dcalls.append(B.PreparedDecode(p, clone, tails, qn, dout, t))
        for i in range(max(args.warmup, ncop)):
            dcalls[i % ncop].run(stream)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record(stream)
        for i in range(args.steps):
            dcalls[i % ncop].run(stream)
        ev1.record(stream)
        torch.cuda.synchronize()
        dec_s = ev0.elapsed_time(ev1) * 1e-3 / args.steps
        dec = {"tail_len": t, "us_per_call": dec_s * 1e6, "layers_per_call": len(layers), "algorithmic_bytes": dec_bytes,
               "achieved_GBps": dec_bytes / dec_s / 1e9, "hbm_frac": dec_bytes / dec_s / HBM_PEAK,
               "cache_copies_round_robin": ncop,
               "note": ("the copies together exceed the 256 MB Infinity Cache" if ncop * dec_bytes > 256 * 2 ** 20
                        else "the copies together still fit the 256 MB Infinity Cache (not the 32 MB of L2)")}
    sim = None
    if args.similarity_block > 0:
        blk = args.similarity_block
        nb = -(-wl.seq_len // blk)
        red = [torch.empty((wl.batch, wl.n_kv_heads), dtype=torch.float32, device=dev) for _ in layers]
        maps = [torch.empty((wl.batch, wl.n_kv_heads, nb, nb), dtype=torch.float32, device=dev) for _ in layers]
        sws = torch.empty(B.mixkv_similarity_workspace_size(p, len(layers), blk), dtype=torch.uint8, device=dev)
        scalls = [B.PreparedSimilarity(p, [x[0] for x in c], red, maps, blk, sws) for c in copies]
        for i in range(args.warmup):
            scalls[i % len(scalls)].run(stream)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record(stream)
        for i in range(args.steps):
            scalls[i % len(scalls)].run(stream)
        ev1.record(stream)
        torch.cuda.synchronize()
        sim_s = ev0.elapsed_time(ev1) * 1e-3 / args.steps
        sim_bytes = units * (wl.seq_len * wl.head_dim * e + nb * nb * 4)          # X once, the map written once
        sim = {"block": blk, "ms_per_call": sim_s * 1e3, "algorithmic_bytes": sim_bytes,
               "achieved_GBps": sim_bytes / sim_s / 1e9, "hbm_frac": sim_bytes / sim_s / HBM_PEAK,
               "kernels": "blocksum_kernel + blockgram_kernel, HIP events on the launch stream"}
    reads_v = args.intrinsic == "vnorm"
    # The other figures the workload definition asks for, from the same process: the fixed budgets
    # 128 / 256 / 512 (cold: the copies of the cache used round-robin) and the default budget warm
    # (one copy, so whatever the chip's caches keep between steps stays).  Each is the median of
    # `steps` event-timed steps after `warmup`.
    sweep = None
    if (not args.no_sweep and args.workload == "c3" and not args.layers and head_budgets is None and not args.given_lse
            and args.intrinsic == "vnorm" and args.mix == "head_adaptive" and wl.budget_mode == "fixed"):
        sweep = {}
        nsteps, nwarm = max(20, args.steps), max(3, args.warmup)

        def figure(bud, cps):
            pb = B.make_params(wl.dtype, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.seq_len, wl.window, bud,
                               pool=wl.pool, pool_kernel=wl.pool_kernel, softmax_scale=wl.softmax_scale, eps=wl.eps,
                               budget_mode="fixed", budget_floor=wl.budget_floor)
            ob = [B.alloc_layer_out(pb, dev, scores=False, redundancy=True) for _ in layers]
            wb = B.alloc_workspace(pb, len(layers), dev)
            cb = [B.PreparedCall(pb, [x[0] for x in c], [x[1] for x in c], [x[2] for x in c], ob, wb) for c in cps]
            wall, per = timed_steps(cb, nsteps, nwarm, stream)
            med = float(np.median(per))
            nbytes = algorithmic_bytes(wl, bud, scores_out=False, reads_v=True) * wl.n_units
            return {"ms_per_step": med, "ms_per_step_wall_mean": wall, "tokens_per_s": wl.batch * wl.seq_len / (med * 1e-3),
                    "hbm_frac_end_to_end": nbytes / (med * 1e-3) / HBM_PEAK, "steps": nsteps, "copies": len(cps)}

        for bud in (128, 256, 512):
            if bud != budget:
                sweep[f"B={bud}"] = figure(bud, copies)
        sweep[f"B={budget}, warm"] = figure(budget, copies[:1])
    bytes_step = algorithmic_bytes(wl, budget, scores_out=False, reads_v=reads_v) * units
    dom = max(("stats", "attn"), key=lambda k: stage_ms.get(k, 0.0))
    kv_bytes = wl.seq_len * wl.head_dim * e
    q_bytes = wl.group * wl.window * wl.head_dim * e
    dom_bytes = ((2 * kv_bytes if dom == "stats" and reads_v else kv_bytes) + q_bytes) * units      # per launch
    dom_s = stage_ms[dom] * 1e-3
    gemm_flops = 2.0 * wl.group * wl.window * wl.seq_len * wl.head_dim * units             # one pass
    out = {
        "metric": "cached tokens compressed/sec (all layers·heads) at 8K ctx; % of HBM peak",
        "value": wl.batch * wl.seq_len / (dt / args.steps),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_stat": "median of the steps, each timed with HIP events on the launch stream",
        "ms_per_step_wall_mean": wall_ms, "ms_per_step_min": float(min(per_step)), "ms_per_step_max": float(max(per_step)),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.n_layers} layers x {wl.n_q_heads}Q/{wl.n_kv_heads}KV heads, D={wl.head_dim}, "
                               f"N={wl.seq_len}, W={wl.window}, B={budget}, batch={wl.batch}, "
                               f"{wl.budget_mode if head_budgets is None else 'per-layer pyramid (mean B)'} budgets, "
                               f"pool=max{wl.pool_kernel}, intrinsic={args.intrinsic}, mix={args.mix}"
                               + (", window log-sum-exp given" if args.given_lse else ""),
                   "units": units, "input_copies_round_robin": len(copies)},
        "hbm_frac_end_to_end": bytes_step / (dt / args.steps) / HBM_PEAK,
        "algorithmic_bytes_per_step": bytes_step,
        "head_tokens_per_s": units * wl.seq_len / (dt / args.steps),
        "stage_ms": {k: round(v, 5) for k, v in stage_ms.items()},
        "mfma_tflops": {k: gemm_flops / (stage_ms[k] * 1e-3) / 1e12 for k in ("stats", "attn") if stage_ms.get(k)},
        "roofline": {"bound": "hbm", "kernel": dom + "_kernel", "achieved": dom_bytes / dom_s / 1e9,
                     "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": dom_bytes / dom_s / HBM_PEAK,
                     "algorithmic_bytes": dom_bytes, "avg_launch_us": dom_s * 1e6,
                     "traffic": (profiled_traffic(args, wl, dom) or {}).get("bytes_per_launch"),
                     "traffic_source": profiled_traffic(args, wl, dom)},
        "cpu_baseline": cpu,
        "other_budgets_and_warm": sweep,
        "similarity": sim,
        "decode": dec,
        "parity_vs_oracle": parity,
        "host_gen_s": round(t_gen, 2),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
