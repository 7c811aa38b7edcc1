#!/usr/bin/env python3
"""Benchmark of the ST3 hot path on one MI355X.

A "step" is one whole job over one batch of synthetic input: prefill of every layer with
progressive visual-token pruning (attention + mass, top-k, stable compaction), then T decode
steps with visual-token annealing (select-and-compact, append, split-KV attention + mass per
layer).  value = generated tokens per second = B*T / job time, inputs resident in HBM.

Prints ONE JSON line: metric, value (tokens/s), timing fields, a `roofline` object for the decode attention
kernel (achieved against the 8 TB/s HBM peak), the unpruned run, KV bytes and a `cpu_baseline` object.
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

HBM_PEAK_GBS = 8000.0
# the roofline pass times the decode attention kernel through the library's diagnostic block
# (st3_profile_*), which is inert unless this is set before the library is loaded
os.environ.setdefault("ST3_DEBUG", "1")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="llava15_13b")
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--decode-steps", type=int, default=0, help="0 = the workload's own T")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-unpruned", action="store_true")
    ap.add_argument("--no-profile-pass", action="store_true")
    ap.add_argument("--no-layer-calls", action="store_true", help="skip the run that makes one library call per layer")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--layer-schedule", default="workload", choices=["workload", "linear", "pvtp", "full"],
                    help="retention over layers: the workload's own, or the paper's strided PVTP (Alg. 1, Eq. 9)")
    ap.add_argument("--stride", type=int, default=4, help="PVTP stride S")
    ap.add_argument("--R-bp", type=int, default=500, help="PVTP ratio R removed per later event, basis points")
    ap.add_argument("--P-bp", type=int, default=5000, help="PVTP ratio P removed at the first event, basis points")
    ap.add_argument("--step-schedule", default="workload", choices=["workload", "cos", "linear", "exp", "none"],
                    help="attenuation over decode steps (Eq. 8 / Sec. 4.4)")
    ap.add_argument("--tau", type=float, default=0.0, help="tau (cos, linear) or sigma (exp); 0 = decode steps")
    ap.add_argument("--lazy", default="",
                    help="QK heredity groups (Eq. 6, Alg. 2) as SRC:FIRST-LAST[,SRC:FIRST-LAST...], e.g. 36:37-39 = "
                         "layers 37..39 reuse the attention probabilities of layer 36 (the paper's '28 -> 29~31' for "
                         "the 7B model); lazy layers take their source's row of the retention table")
    ap.add_argument("--contiguous-tail", action="store_true",
                    help="keep every cache contiguous (an eviction closes the tail up: two row moves per evicted row) "
                         "instead of leaving the instruction + generated rows at a fixed offset (one move)")
    ap.add_argument("--kv-format", default="plain", choices=["plain", "e4m3"],
                    help="e4m3: the KV caches hold FP8 E4M3 codes with one scale per (b, h) strip (6 sigma / 448); an extra "
                         "configuration beside the bf16 headline, not part of the paper")
    ap.add_argument("--length-probe", type=int, default=0, metavar="BLOCK",
                    help="decode latency and KV bytes against the generated length (the paper's latency figure, right "
                         "panel): times every BLOCK decode steps of one job, pruned and unpruned; prints one JSON object")
    ap.add_argument("--graph-probe", type=int, default=0, metavar="CHUNK",
                    help="side mode: decode steps launched one by one against the same steps replayed from HIP graphs "
                         "captured CHUNK steps at a time")
    ap.add_argument("--prefill-probe", action="store_true",
                    help="prefill only (all layers with progressive pruning), three passes, for kernel traces and MFMA "
                         "counters of the prefill attention kernel; prints each layer's length and algorithmic flops")
    ap.add_argument("--attend-tile", type=int, default=0, metavar="U",
                    help="force one build of the decode attention kernel (16-byte loads per lane and tile: 1, 4, 6, 8; "
                         "E4M3 caches: 1, 3, 4) instead of the launcher's own choice per launch; 0 = automatic")
    ap.add_argument("--select-probe", action="store_true",
                    help="time the selection and compaction calls alone (top-k, in-place eviction in both modes and both "
                         "cache layouts, the prefill gather) at the workload's shape and print one JSON line")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="short run for counter collection: prefill, one plain 1 GiB device copy of known size, "
                         "then the decode steps; prints the algorithmic bytes of each attend launch")
    return ap.parse_args()


class Job:
    """Device-resident inputs of one batch and the call sequence of one whole job."""

    def __init__(self, w, B, T, keep, torch, pipeline, st3, seed=1234, lazy=None, kv_format="plain", fixed_tail=True):
        self.w, self.B, self.T, self.keep = w, B, T, keep
        self.lazy = dict(lazy or {})
        self.kv_format = kv_format
        self.torch = torch
        dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        dev = "cuda:0"
        g = torch.Generator(device=dev)
        g.manual_seed(seed)
        shape_p = (B, w.heads, w.n_prompt, w.head_dim)
        shape_d = (w.layers, 3, B, w.heads, w.head_dim)

        def randn(shape):
            return (torch.randn(shape, generator=g, device=dev, dtype=torch.float32) * w.sigma).to(dt)

        self.pre = [tuple(randn(shape_p) for _ in range(3)) for _ in range(w.layers)]
        self.dec = [randn(shape_d) for _ in range(T)]
        self.gen = pipeline.Generation(w.layers, w.heads, w.head_dim, dt, B, w.n_sys, w.n_vis, w.n_txt, T, keep,
                                       device=dev, lazy=self.lazy,
                                       kv_scale=(6 * w.sigma / 448) if kv_format == "e4m3" else None,
                                       fixed_tail=fixed_tail)

    def run(self):
        gen, w = self.gen, self.w
        for l in range(w.layers):
            q, k, v = self.pre[l]
            gen.prefill_layer(l, q, k, v)
        for t in range(1, self.T + 1):
            gen.decode_step(t, self.dec[t - 1])

    def run_layer_calls(self):
        """The same job through the calls a decoder with a dependency between its layers can make:
        st3_decode_layer_attend once per layer (each could wait for the previous layer's output),
        then st3_decode_plans once per step."""
        gen, w = self.gen, self.w
        for l in range(w.layers):
            q, k, v = self.pre[l]
            gen.prefill_layer(l, q, k, v)
        one = self.B * w.heads * w.head_dim * self.dec[0].element_size()        # bytes of one [B,H,d] input
        for t in range(1, self.T + 1):
            base = self.dec[t - 1].data_ptr()                                   # [L, 3, B, H, d]: q, k_new, v_new per layer
            gen.begin_step(t)
            for l in range(w.layers):
                gen.attend_layer(l, base + 3 * l * one, base + (3 * l + 1) * one, base + (3 * l + 2) * one)
            gen.finish_step()

    def run_prefill_only(self):
        gen, w = self.gen, self.w
        for l in range(w.layers):
            q, k, v = self.pre[l]
            gen.prefill_layer(l, q, k, v)

    def decode_kernel_bytes(self):
        """Algorithmic HBM bytes of all split-KV decode launches of one job: per (sequence, layer,
        step) K and V rows read once, plus q in, o out and the mass row."""
        w = self.w
        e = 2 if w.dtype == "bf16" else 4
        ekv = 1 if self.kv_format == "e4m3" else e
        total = 0
        for t in range(1, self.T + 1):
            for l in range(w.layers):
                if l in self.lazy:          # a lazy layer runs the V-only kernel, not this one
                    continue
                lkv = w.n_sys + self.keep[l][t] + w.n_txt + t
                total += self.B * (2 * w.heads * w.head_dim * ekv * lkv + 2 * w.heads * w.head_dim * e
                                   + 4 * self.keep[l][t])
        return total


def committed_traffic(workload, batch, kv_format, alg_bytes_per_launch):
    """HBM bytes per launch of the decode attention kernel from the committed counter summary
    (two `rocprofv3 --pmc` runs, FETCH_SIZE then WRITE_SIZE, calibrated by a copy of known size):
    that run's traffic / algorithmic ratio times this run's algorithmic bytes per launch.  Not
    measured in this run (counters need the profiler attached): None when no summary covers the
    workload, and the source is always named next to the number."""
    tag = f"{workload}_b{batch}" + ("" if kv_format == "plain" else f"_{kv_format}")
    path = os.path.join("profiles", f"decode_attend_kernel_{tag}_pmc.txt")
    try:
        with open(os.path.join(ROOT, path)) as f:
            for line in f:
                if line.startswith("traffic / algorithmic ="):
                    ratio = float(line.split("=")[1].split()[0])
                    return ratio * alg_bytes_per_launch, (f"not measured in this run: ratio {ratio} of the committed "
                                                          f"rocprofv3 --pmc summary {path} x this run's algorithmic bytes")
    except (OSError, ValueError, IndexError):
        pass
    return None, "no committed rocprofv3 --pmc summary covers this workload"


def timed(torch, fn, reps):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / reps


def cpu_baseline(w, keep, T, budget_s):
    """The oracle (NumPy fp64, as it stands) on the host cores: its decode step at B = 1 on sampled
    steps of the same workload, once with the BLAS pool at the cores this process may use and once
    on one thread; the tiny workload is timed in full (prefill + all decode steps)."""
    import numpy as np
    from threadpoolctl import threadpool_info, threadpool_limits

    from oracle import st3_oracle as orc
    nproc = os.cpu_count() or 1
    try:
        usable = len(os.sched_getaffinity(0))
    except (AttributeError, OSError):
        usable = nproc
    want = max(1, min(usable, int(os.environ.get("OMP_NUM_THREADS", usable) or usable)))
    rng = np.random.default_rng(0)
    sample_steps = sorted(set([1, max(1, T // 4), max(1, T // 2), max(1, 3 * T // 4), T]))

    def one_step(t):
        g = orc.Generation(w.layers, w.heads, w.head_dim, w.n_sys, w.n_vis, w.n_txt, np.array(keep))
        for l in range(w.layers):
            nv = keep[l][t - 1]
            n = w.n_sys + nv + w.n_txt + (t - 1)
            g.K.append([rng.standard_normal((w.heads, n, w.head_dim))])
            g.V.append([rng.standard_normal((w.heads, n, w.head_dim))])
            g.ids.append([np.arange(nv, dtype=np.int64)])
            g.rho.append([rng.random(nv)])
        g.t = t - 1
        qkv = [tuple(rng.standard_normal((1, w.heads, w.head_dim)) for _ in range(3)) for _ in range(w.layers)]
        t0 = time.perf_counter()
        g.decode_step(lambda l: qkv[l])
        return time.perf_counter() - t0

    def whole_job():
        g = orc.Generation(w.layers, w.heads, w.head_dim, w.n_sys, w.n_vis, w.n_txt, np.array(keep))
        shape_p = (1, w.heads, w.n_prompt, w.head_dim)
        pre = [tuple(rng.standard_normal(shape_p) for _ in range(3)) for _ in range(w.layers)]
        dec = [[tuple(rng.standard_normal((1, w.heads, w.head_dim)) for _ in range(3)) for _ in range(w.layers)]
               for _ in range(T)]
        t0 = time.perf_counter()
        g.prefill(lambda l: pre[l])
        for t in range(T):
            g.decode_step(lambda l: dec[t][l])
        return time.perf_counter() - t0

    def measure(threads, budget):
        with threadpool_limits(limits=threads):
            pools = [p.get("num_threads", 1) for p in threadpool_info()]
            used = max(pools) if pools else 1
            spent, times = 0.0, []
            reps = 0
            while spent < budget and reps < 50:
                if w.name == "tiny":
                    dt = whole_job(); times.append(dt); spent += dt
                else:
                    for t in sample_steps:
                        dt = one_step(t); times.append(dt); spent += dt
                reps += 1
        mean = sum(times) / len(times)
        per_token = mean / T if w.name == "tiny" else mean      # seconds per generated token at B = 1
        return {"value": 1.0 / per_token, "cores": used, "timed": len(times), "seconds": round(spent, 1)}

    many = measure(want, budget_s / 2)
    one = measure(1, budget_s / 2)
    what = (f"whole job (prefill + {T} decode steps) at B=1, {many['timed']} runs" if w.name == "tiny" else
            f"B=1, oracle decode step (all {w.layers} layers: evict, append, attention, mass) at steps t in {sample_steps} "
            f"of {w.name}, {many['timed']} timed steps; prefill excluded")
    return {"value": many["value"], "unit": "tokens/s", "cores": many["cores"], "kind": "oracle",
            "sample": f"{what}, {many['seconds']} s on {many['cores']} BLAS threads (host reports {nproc} CPUs, {usable} usable) "
                      f"and {one['seconds']} s on 1 thread; cost is linear in B",
            "one_core": {"value": one["value"], "unit": "tokens/s", "cores": 1, "timed": one["timed"]},
            "host_cpus": nproc, "usable_cpus": usable}


def pmc_probe(a, w, B, T, keep, torch, pipeline, st3, lazy=None):
    """For `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE`: the same decode launches as the
    benchmark (first T steps), preceded by a device-to-device copy of exactly 1 GiB whose counter
    reading calibrates the counter's unit."""
    lazy = dict(lazy or {})
    job = Job(w, B, T, keep, torch, pipeline, st3, lazy=lazy, kv_format=a.kv_format, fixed_tail=not a.contiguous_tail)
    job.run_prefill_only()
    n = 1 << 30
    src = torch.empty((n,), dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    src.fill_(1)
    torch.cuda.synchronize()
    dst.copy_(src)                  # the calibration kernel: reads 1 GiB, writes 1 GiB
    torch.cuda.synchronize()
    for t in range(1, T + 1):
        job.gen.decode_step(t, job.dec[t - 1])
    torch.cuda.synchronize()
    e = 2 if w.dtype == "bf16" else 4
    per_launch, per_lazy = [], []
    hd = w.heads * w.head_dim * e
    hd_kv = w.heads * w.head_dim * (1 if a.kv_format == "e4m3" else e)      # one cached row over all heads
    for t in range(1, T + 1):
        for l in range(w.layers):
            lkv = w.n_sys + keep[l][t] + w.n_txt + t
            if l in lazy:       # V rows once, one logit per (head, key), v_new in, o out
                per_lazy.append(B * (hd_kv * lkv + 4 * w.heads * lkv + 2 * hd))
            else:
                per_launch.append(B * (2 * hd_kv * lkv + 2 * hd + 4 * keep[l][t]))
    print(json.dumps({"probe": "pmc", "workload": w.name, "batch": B, "decode_steps": T, "kv_format": a.kv_format,
                      "copy_bytes_read": n, "copy_bytes_written": n,
                      "attend_launches": len(per_launch), "alg_bytes_per_launch_mean": sum(per_launch) / len(per_launch),
                      "alg_bytes_first_launches": per_launch[:8],
                      "inherit_launches": len(per_lazy),
                      "inherit_alg_bytes_per_launch_mean": (sum(per_lazy) / len(per_lazy)) if per_lazy else None}))


def length_probe(w, B, T, keep, block, lazy, kv_format, torch, pipeline, st3):
    """Per block of decode steps: mean ms per step and KV bytes held at the end of the block, for the
    pruned schedule and for the same kernels without pruning."""
    import dataclasses
    wu = dataclasses.replace(w, layer_schedule={"kind": "full"}, step_schedule={"kind": "none"})
    keep_u = [row[:T + 1] for row in pipeline.keep_table_for(wu)]
    out = {"probe": "length", "workload": w.name, "batch": B, "decode_steps": T, "block": block, "rows": []}
    series = {}
    shared = None
    for name, kp, lz in (("pruned", keep, lazy), ("unpruned", keep_u, {})):
        job = Job(w if name == "pruned" else wu, B, T, kp, torch, pipeline, st3, lazy=lz, kv_format=kv_format)
        if shared is not None:
            job.pre, job.dec = shared
        shared = (job.pre, job.dec)
        job.run()                                   # warm-up
        job.run_prefill_only()
        torch.cuda.synchronize()
        rows = []
        for t0 in range(1, T + 1, block):
            t1 = min(t0 + block, T + 1)
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            for t in range(t0, t1):
                job.gen.decode_step(t, job.dec[t - 1])
            torch.cuda.synchronize()
            rows.append({"generated": t1 - 1, "ms_per_step": (time.perf_counter() - c0) * 1e3 / (t1 - t0),
                         "kv_bytes": job.gen.kv_bytes()})
        series[name] = rows
        del job
        torch.cuda.empty_cache()
    for a_, b_ in zip(series["pruned"], series["unpruned"]):
        out["rows"].append({"generated": a_["generated"], "pruned_ms_per_step": a_["ms_per_step"],
                            "unpruned_ms_per_step": b_["ms_per_step"], "pruned_kv_bytes": a_["kv_bytes"],
                            "unpruned_kv_bytes": b_["kv_bytes"]})
    print(json.dumps(out))


def graph_probe(w, B, T, keep, chunk, lazy, kv_format, torch, pipeline, st3):
    """Decode steps issued call by call against the same launch sequence replayed from HIP graphs.  A graph
    holds the launches of `chunk` consecutive steps with those steps' scalars (bounds, keep counts, input
    addresses) baked in, so it serves any later job of the same shape and schedule whose inputs sit in the
    same buffers.  Every replayed job is compared with the eager one (outputs of the last step, lengths)."""
    job = Job(w, B, T, keep, torch, pipeline, st3, lazy=lazy, kv_format=kv_format)
    gen = job.gen
    job.run()                                       # warm-up, fills the library's per-device caches
    torch.cuda.synchronize()

    def lengths():
        return [(lc.vis_len.clone(), lc.kv_len.clone()) for lc in gen.layers]

    def timed_decode(step_fn):
        job.run_prefill_only()
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        step_fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - c0) * 1e3 / T

    def eager():
        for t in range(1, T + 1):
            gen.decode_step(t, job.dec[t - 1])

    eager_ms = min(timed_decode(eager) for _ in range(3))
    ref_out, ref_len = gen.dec_out_all.clone(), lengths()
    # capture: nothing runs, the host-side bookkeeping of the pipeline advances as in a real job
    job.run_prefill_only()
    torch.cuda.synchronize()
    graphs = []
    for t0 in range(1, T + 1, chunk):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for t in range(t0, min(t0 + chunk, T + 1)):
                gen.decode_step(t, job.dec[t - 1])
        graphs.append(g)
    torch.cuda.synchronize()

    def replay():
        for g in graphs:
            g.replay()

    graph_ms, same = [], True
    for _ in range(3):
        graph_ms.append(timed_decode(replay))
        same = same and bool(torch.equal(gen.dec_out_all, ref_out))
        for (v0, k0), (v1, k1) in zip(ref_len, lengths()):
            same = same and bool(torch.equal(v0, v1)) and bool(torch.equal(k0, k1))
        _ = timed_decode(eager)                     # eager work between the replayed jobs
        same = same and bool(torch.equal(gen.dec_out_all, ref_out))
    print(json.dumps({"probe": "graph", "workload": w.name, "batch": B, "decode_steps": T, "chunk": chunk,
                      "graphs": len(graphs), "eager_ms_per_step": eager_ms, "graph_ms_per_step": min(graph_ms),
                      "graph_ms_per_step_all": graph_ms, "replays_match_eager": same}))
    return 0 if same else 1


def prefill_probe(w, B, keep, torch, pipeline, st3):
    """Three prefill passes; per layer: tokens attended and algorithmic flops (causal half of QK^T and PV)."""
    job = Job(w, B, 1, [row[:2] for row in keep], torch, pipeline, st3)
    for _ in range(3):
        job.run_prefill_only()
    torch.cuda.synchronize()
    ms = timed(torch, job.run_prefill_only, 3) * 1e3
    layers = []
    for l in range(w.layers):
        n_l = w.n_sys + keep[l][0] + w.n_txt
        layers.append({"layer": l, "n": n_l, "flops": B * 4 * w.heads * w.head_dim * n_l * (n_l + 1) // 2})
    print(json.dumps({"probe": "prefill", "workload": w.name, "batch": B, "prefill_ms_all_layers": ms,
                      "flops_all_layers": sum(x["flops"] for x in layers), "layers": layers}))


def select_probe(w, B, torch, st3):
    """Selection and compaction on their own (the steps between two attentions): microseconds per call
    from a start/stop event pair around each call, and the bytes the call has to move."""
    dev = torch.device("cuda:0")
    H, d, ns, nv, nx = w.heads, w.head_dim, w.n_sys, w.n_vis, w.n_txt
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    eb = 2 if w.dtype == "bf16" else 4
    shape = st3.make_shape(B, H, d, st3.ST3_BF16 if w.dtype == "bf16" else st3.ST3_F32)
    gen = 64                                    # generated rows behind the prompt
    n0 = ns + nv + nx + gen
    cap = n0 + 8
    K = torch.randn((B, H, cap, d), device=dev).to(dt); V = torch.randn((B, H, cap, d), device=dev).to(dt)
    ws = torch.empty((st3.st3_workspace_bytes(shape, cap, nv, 1),), dtype=torch.uint8, device=dev)
    st3.st3_workspace_init(shape, cap, ws)
    score0 = torch.rand((B, nv), device=dev)
    ids0 = torch.arange(nv, device=dev, dtype=torch.int32).repeat(B, 1).contiguous()
    score, ids = score0.clone(), ids0.clone()
    vis_len = torch.empty((B,), dtype=torch.int32, device=dev); kv_len = torch.empty_like(vis_len)
    tail = torch.full((B,), ns + nv, dtype=torch.int32, device=dev)
    kv = st3.kv_layer(K, V)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def one(fn, reset, reps=12):
        """Microseconds per call.  reset=None: the call leaves no state behind, so `reps` calls run back to
        back between one pair of events.  Otherwise every call gets its own pair (after `reset`), which adds
        the cost of the pair itself: the row with evicted = 0 shows that floor."""
        tot = 0.0
        if reset is None:
            fn(); fn()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                fn()
            e1.record(); torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps * 1e3
        for r in range(reps + 2):
            reset()
            e0.record(); fn(); e1.record()
            torch.cuda.synchronize()
            if r >= 2:
                tot += e0.elapsed_time(e1)
        return tot / reps * 1e3

    # one plain device-to-device copy of exactly 1 GiB: what FETCH_SIZE / WRITE_SIZE read for it calibrates
    # those counters when this probe runs under rocprofv3 --pmc
    cal_src = torch.empty((1 << 30,), dtype=torch.uint8, device=dev); cal_dst = torch.empty_like(cal_src)
    cal_src.fill_(1); torch.cuda.synchronize(); cal_dst.copy_(cal_src); torch.cuda.synchronize()
    del cal_src, cal_dst
    rows = []
    # top-k alone (Eq. 3): scores of one prune event
    mask = torch.empty((B, nv), dtype=torch.uint8, device=dev)
    for k in sorted({nv // 2, nv // 10}):
        idx = torch.empty((B, k), dtype=torch.int32, device=dev)
        us = one(lambda: st3.st3_select_topk(score0, ids0, None, nv, k, mask, idx), None)
        rows.append({"call": "st3_select_topk", "n": nv, "k": k, "us": us, "bytes": B * (8 * nv + nv + 4 * k)})
    # eviction of e visual rows from one layer's cache (Eq. 7, Sec. 4.3), both modes, both layouts
    row_bytes = 2 * H * d * eb                  # one cache row of a sequence, K and V over all heads
    for e in (0, 1, 4, 16, 64, nv // 2):
        for mode, mname in ((st3.ST3_HOLE_FILL, "hole_fill"), (st3.ST3_STABLE, "stable")):
            for fixed in (False, True):
                def reset():
                    score.copy_(score0); ids.copy_(ids0); vis_len.fill_(nv); kv_len.fill_(n0)
                seg = st3.segments(ns, nv, n0, vis_len, kv_len, tail if fixed else None, nv, ns + nv if fixed else 0)
                us = one(lambda: st3.st3_select_compact_layer(shape, kv, seg, score, ids, nv - e, mode, ws), reset)
                # rows moved, summed over the batch, from the scores (victims = the e lowest scores of a sequence)
                if e == 0:
                    moved = 0
                else:
                    victim = torch.zeros((B, nv), dtype=torch.bool, device=dev)
                    victim.scatter_(1, score0.argsort(dim=1)[:, :e], True)
                    if mode == st3.ST3_HOLE_FILL:   # survivors in the last e places of the segment fill the holes in front of them
                        moved = int((~victim[:, nv - e:]).sum().item()) + (0 if fixed else B * min(e, nx + gen))
                    else:                           # every surviving row behind a sequence's first hole is rewritten
                        first = victim.float().argmax(dim=1)
                        moved = int((nv - first).sum().item()) - B * e + (0 if fixed else B * (nx + gen))
                rows.append({"call": "st3_select_compact_layer", "mode": mname, "tail": "fixed" if fixed else "contiguous",
                             "evicted": e, "us": us, "bytes": 2 * moved * row_bytes})
    # the prefill gather (Alg. 1: X = [S, V_kept, I]) of a layer's Q, K, V rows
    n_all = ns + nv + nx
    src = [torch.randn((B, H, n_all, d), device=dev).to(dt) for _ in range(3)]
    for k in sorted({nv // 2, nv // 10}):
        dst = [torch.empty((B, H, ns + k + nx, d), device=dev, dtype=dt) for _ in range(3)]
        idx = torch.sort(torch.rand((B, nv), device=dev).argsort(dim=1)[:, :k].to(torch.int32), dim=1).values.contiguous()
        us = one(lambda: st3.st3_gather_rows(list(zip(src, dst)), ns, idx, k, nv, nx), None)
        rows.append({"call": "st3_gather_rows", "tensors": 3, "n": nv, "k": k, "us": us,
                     "bytes": 2 * 3 * B * H * (ns + k + nx) * d * eb})
    for r in rows:
        r["GBps"] = r["bytes"] / (r["us"] * 1e-6) / 1e9
    print(json.dumps({"probe": "select", "workload": w.name, "batch": B, "cache_rows": n0, "rows": rows}))


def main():
    a = parse()
    if a.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (every box has one); --gpus {a.gpus} is not supported",
              file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2412_20105_amd import binding as st3
    from paper_2412_20105_amd import pipeline
    from workloads import get_workload
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    st3.lib()                                   # fail loudly if the library is not built
    w = get_workload(a.workload)
    T = a.decode_steps or w.steps
    import dataclasses
    if a.layer_schedule == "pvtp":
        w = dataclasses.replace(w, layer_schedule={"kind": "pvtp", "S": a.stride, "P_bp": a.P_bp, "R_bp": a.R_bp})
    elif a.layer_schedule == "full":
        w = dataclasses.replace(w, layer_schedule={"kind": "full"})
    elif a.layer_schedule == "linear":
        w = dataclasses.replace(w, layer_schedule={"kind": "linear", "last_full_layer": 2, "end_ratio_bp": 1000})
    if a.step_schedule != "workload":
        par = a.tau or float(T)
        ss = {"cos": {"kind": "cos", "tau": par}, "linear": {"kind": "linear", "tau": par},
              "exp": {"kind": "exp", "sigma": par}, "none": {"kind": "none"}}[a.step_schedule]
        w = dataclasses.replace(w, step_schedule=ss)
    w = dataclasses.replace(w, steps=T)
    B = a.batch
    keep = [row[:T + 1] for row in pipeline.keep_table_for(w)]
    lazy = {}
    for grp in filter(None, a.lazy.split(",")):
        src, rng = grp.split(":")
        first, last = (rng.split("-") + [rng])[:2]
        for l in range(int(first), int(last) + 1):
            lazy[l] = int(src)
            keep[l] = list(keep[int(src)])          # a lazy layer holds what its source holds
    def note(msg):
        print(f"[bench] {msg}", file=sys.stderr, flush=True)

    if a.attend_tile:
        st3.st3_debug_set_attend_tile(a.attend_tile)
    if a.select_probe:
        return select_probe(w, B, torch, st3)
    if a.prefill_probe:
        return prefill_probe(w, B, keep, torch, pipeline, st3)
    if a.graph_probe:
        return graph_probe(w, B, T, keep, a.graph_probe, lazy, a.kv_format, torch, pipeline, st3)
    if a.length_probe > 0:
        return length_probe(w, B, T, keep, a.length_probe, lazy, a.kv_format, torch, pipeline, st3)
    if a.pmc_probe:
        return pmc_probe(a, w, B, T, keep, torch, pipeline, st3, lazy)

    note(f"generating inputs for {w.name} B={B} T={T}")
    job = Job(w, B, T, keep, torch, pipeline, st3, lazy=lazy, kv_format=a.kv_format, fixed_tail=not a.contiguous_tail)
    note("warmup")
    for _ in range(a.warmup):
        job.run()
    torch.cuda.synchronize()
    note("timed region")
    ms_job = timed(torch, job.run, a.steps) * 1e3
    tokens = B * T
    value = tokens / (ms_job * 1e-3)
    ms_prefill = timed(torch, job.run_prefill_only, 1) * 1e3
    kv_bytes_end = job.gen.kv_bytes() if False else None

    result = {
        "metric": "pruned decode attention tokens/s + HBM GB/s (% peak), LLaVA-1.5-13B shape",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_job, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: L={w.layers} H={w.heads} d={w.head_dim} {w.dtype}, prompt "
                               f"{w.n_sys}+{w.n_vis}+{w.n_txt}, T={T} decode steps, batch {B}, "
                               f"schedule {w.layer_schedule}/{w.step_schedule}",
                   "batch": B, "decode_steps": T, "step_definition": "prefill (all layers, PVTP) + T decode steps (VTA)",
                   "lazy_layers": {str(l): s for l, s in sorted(lazy.items())}, "kv_format": a.kv_format,
                   "tail": "contiguous" if a.contiguous_tail else "fixed offset",
                   "attend_tile": a.attend_tile or "automatic"},
        "prefill_ms": ms_prefill,
        "decode_ms_per_token_step": (ms_job - ms_prefill) / T,
        "decode_only_tokens_per_s": tokens / ((ms_job - ms_prefill) * 1e-3),
    }

    # -- the same job through one library call per layer (what a real decoder can call) -----------
    if not a.no_layer_calls:
        note("per-layer calls")
        job.run_layer_calls()
        ms_lc = timed(torch, job.run_layer_calls, 1) * 1e3
        result["per_layer_calls"] = {
            "value": tokens / (ms_lc * 1e-3), "unit": "tokens/s", "ms_per_step": ms_lc,
            "decode_ms_per_token_step": (ms_lc - ms_prefill) / T,
            "calls": "st3_decode_layer_attend per layer + st3_decode_plans per step (the headline uses st3_decode_step: "
                     "the same launches from one host call per step)"}

    # -- roofline of the dominant kernel (split-KV decode), from a second, instrumented pass ---------
    note(f"job {ms_job:.1f} ms, prefill {ms_prefill:.1f} ms")
    if not a.no_profile_pass:
        note("instrumented pass")
        launches = (w.layers - len(lazy)) * T
        st3.st3_profile_enable(launches + 8)
        job.run()
        torch.cuda.synchronize()
        tot_ms, cnt, mn, mx = st3.st3_profile_read()
        alg = job.decode_kernel_bytes()
        achieved = alg / (tot_ms * 1e-3) / 1e9 if tot_ms > 0 else 0.0
        traffic, traffic_source = committed_traffic(w.name, B, a.kv_format, alg / max(cnt, 1))
        result["roofline"] = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                              "kernel": "decode_attend_kernel", "launches": cnt,
                              "avg_launch_us": tot_ms * 1e3 / max(cnt, 1), "min_us": mn * 1e3, "max_us": mx * 1e3,
                              "alg_bytes_per_launch": alg / max(cnt, 1),
                              "kernel_time_share_of_job": tot_ms / ms_job}
        result["kv_bytes_after_last_step"] = job.gen.kv_bytes()

    # -- the same kernels without pruning ---------------------------------------------------------------
    if not a.no_unpruned:
        note("unpruned run")
        wu = dataclasses.replace(w, layer_schedule={"kind": "full"}, step_schedule={"kind": "none"})
        keep_u = [row[:T + 1] for row in pipeline.keep_table_for(wu)]
        del job.gen
        torch.cuda.empty_cache()
        job_u = Job(wu, B, T, keep_u, torch, pipeline, st3, kv_format=a.kv_format, fixed_tail=not a.contiguous_tail)
        job_u.pre, job_u.dec = job.pre, job.dec
        job_u.run()
        ms_u = timed(torch, job_u.run, 1) * 1e3
        result["unpruned"] = {"value": tokens / (ms_u * 1e-3), "unit": "tokens/s", "ms_per_step": ms_u,
                              "kv_bytes_after_last_step": job_u.gen.kv_bytes()}
        result["speedup_vs_unpruned"] = ms_u / ms_job
        if "kv_bytes_after_last_step" in result:
            result["kv_bytes_ratio_vs_unpruned"] = result["kv_bytes_after_last_step"] / job_u.gen.kv_bytes()

    if not a.no_cpu_baseline:
        note("cpu baseline (oracle)")
        result["cpu_baseline"] = cpu_baseline(w, keep, T, a.cpu_seconds)
    result["context"] = "paper headline (A100, whole model): ~2x faster inference at ~30% KV cache vs LLaVA; not a target"
    print(json.dumps(result))


if __name__ == "__main__":
    main()
