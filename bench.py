#!/usr/bin/env python3
"""Benchmark of the Loki decode-attention hot path on one MI355X.

One "step" is one pass of the whole path (query rotation + low-rank scoring, top-k select,
gather attention, combine) over one batch of synthetic input resident in HBM.  The workload
is the Llama-2-7B-shaped configuration (batch 16, 32 heads, D=128, S=4096, bf16, d=32,
k=1024) unless --workload names another one.  Prints ONE JSON line.

Timed region: W warm-up steps, then exactly K steps between two device synchronisations;
consecutive steps use different copies of the KV cache so that no step finds its rows in
the 256 MB last-level cache.  A second pass of K steps records HIP events around every
kernel (on the launch stream, through the library's profile hook) to find the dominant kernel;
the dense baseline is timed the same way.  When the step is a single kernel, the roofline
takes its launch duration from two events on the launch stream around K back-to-back launches.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic.md")


def recorded_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` on `workload` as recorded in profiles/hbm_traffic.md
    (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by the plain-copy calibration; the file names the
    commands and the commit of the kernel sources it was taken at).  Not measured by this run:
    None when the table has no row for the pair."""
    try:
        rows = open(TRAFFIC_TABLE).read().splitlines()
    except OSError:
        return None, None
    for line in rows:
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 5 and cells[0] == workload and cells[1] == kernel:
            try:
                return float(cells[2]) + float(cells[3]), cells[4]
            except ValueError:
                return None, None
    return None, None


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def algorithmic_bytes(w, select_mode):
    """Bytes the method itself must move (Section 4.2 cost model in bytes): the low-rank slab
    once per KV unit plus k full K and V rows per selecting head."""
    e = w.elem_bytes
    units = w.B * w.Hkv
    sel_heads = units if (select_mode == 1 or w.G == 1) else w.B * w.Hq
    score = units * w.S * w.d * e
    gather = sel_heads * w.k * 2 * w.D * e
    dense = units * w.S * 2 * w.D * e
    return {"score": score, "gather_attend": gather, "step": score + gather,
            "fused_decode": score + gather, "dense_attend": dense}


def cpu_baseline(w, x, select_mode, budget_s=20.0):
    """The oracle as it stands, timed on the host on a bounded sample of (batch, KV head)
    units of the same workload, scaled to the full unit count."""
    from oracle import loki_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    units = [(b, h) for b in range(w.B) for h in range(w.Hkv)]
    t0 = time.perf_counter()
    done = 0
    while True:  # whole passes over the units until ~budget_s/2 has gone by, then stop
        for u in units:
            O.loki_decode_batch(x["q"], x["P"], x["khat"], x["v"], w.d, w.k, select_mode, units=[u])
            done += 1
            if time.perf_counter() - t0 > budget_s:
                break
        if time.perf_counter() - t0 > budget_s / 2:
            break
    dt = time.perf_counter() - t0
    us_per_step = dt / done * len(units) * 1e6
    return {"value": us_per_step, "unit": "us/step", "cores": int(cores), "kind": "oracle",
            "sample": f"{done} (batch, KV head) unit evaluations of {w.name} "
                      f"({len(units)} units per step) in {dt:.1f} s, scaled to one step"}

def _pct(samples, q):
    return float(np.percentile(np.asarray(samples, dtype=np.float64), q))


def event_timed_steps(torch, step_fn, steps, warmup, stream):
    """Durations of `steps` back-to-back steps, each from one event on the launch stream to the
    next, in microseconds, after `warmup` untimed steps (and at least 30 ms of them)."""
    t_w = time.perf_counter()
    i = 0
    while i < warmup or time.perf_counter() - t_w < 0.03:
        step_fn(i)
        i += 1
        if i % 50 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    evs[0].record(stream)
    for i in range(steps):
        step_fn(i)
        evs[i + 1].record(stream)
    torch.cuda.synchronize()
    wall_us = (time.perf_counter() - t0) / steps * 1e6
    per_step = [evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(steps)]
    return per_step, wall_us


def kernel_times(api, step_fn, steps):
    """Mean HIP-event time of every kernel of a step, microseconds, in launch order (the
    library's profile hook; every launch is read back before the next, so each bracket holds
    one kernel on an otherwise idle device plus about 2.5 us of event overhead)."""
    prof = api.Profile()
    acc, order = {}, []
    prof.attach()
    try:
        for i in range(steps):
            step_fn(i)
            for name, ms in prof.read():
                if name not in acc:
                    acc[name] = []
                    order.append(name)
                acc[name].append(ms)
    finally:
        api.Profile.detach()
        prof.close()
    return {n: float(np.mean(acc[n])) * 1e3 for n in order}


def bench_configs(args, torch, api, synth):
    """The `configs` array: every other workload of the benchmark list, both select modes where
    query heads are grouped, the nine (d, k) points of the large-model sweep, and the benchmark
    workload at batch 1 and 2.  Inputs come
    from the same seeded generator as the parity tests; a workload's cache is generated once and
    the low-rank / residual split is rebuilt on the device per d."""
    cfgs = synth.paper_configs()
    # (the benchmark workload at batch 1 and 2, 32 and 64 units, shows where few units leave every
    # path bound by latency: dense attention has no dependent stages and can be the faster one there)
    small = [cfgs["llama2_7b"].replace(B=b, name=f"llama2_7b_batch{b}") for b in (1, 2)]
    plan = [("tiny", cfgs["tiny"], [cfgs["tiny"]], (0,)),
            ("llama2_7b_batch1", small[0], [small[0]], (0,)),
            ("llama2_7b_batch2", small[1], [small[1]], (0,)),
            ("llama3_8b_gqa", cfgs["llama3_8b_gqa"], [cfgs["llama3_8b_gqa"]], (0, 1)),
            ("long_gqa", cfgs["long_gqa"], [cfgs["long_gqa"]], (0, 1)),
            ("large_share", cfgs["large_share"], synth.large_share_sweep(), (0, 1))]
    stream = torch.cuda.current_stream()
    steps = max(20, args.config_steps)
    entries = []
    for name, base, variants, modes in plan:
        tdt = torch.float32 if base.dtype == "f32" else torch.bfloat16
        t0 = time.perf_counter()
        x = synth.make_inputs(base, threads=min(16, os.cpu_count() or 8))
        kh = torch.from_numpy(x["khat"]).to("cuda").to(tdt)
        vv = torch.from_numpy(x["v"]).to("cuda").to(tdt)
        q = torch.from_numpy(x["q"]).to("cuda").to(tdt)
        P = torch.from_numpy(x["P"]).to("cuda")
        del x
        cache_bytes = 2 * kh.numel() * kh.element_size()
        copies = 2 if cache_bytes >= (1 << 30) else 4  # steps alternate between copies of the cache
        kfs = [kh] + [kh.clone() for _ in range(copies - 1)]
        vs = [vv] + [vv.clone() for _ in range(copies - 1)]
        log(f"[bench] {name}: inputs + upload {time.perf_counter() - t0:.1f} s, {copies} cache copies")
        out = torch.empty((base.B, base.Hq, base.D), dtype=tdt, device="cuda")
        lay0 = api.make_layout(base.B, base.Hq, base.Hkv, base.D, base.d, base.S, tdt)
        wsd = torch.empty(max(api.loki_workspace_bytes(lay0, base.S, 0, 0, -1), 256),
                          dtype=torch.uint8, device="cuda")

        def dense_step(i):
            api.dense_decode_attn(lay0, q, kfs[i % copies], vs[i % copies], base.S, wsd, out, stream)

        d_us, d_wall = event_timed_steps(torch, dense_step, steps, 10, stream)
        dense_us = _pct(d_us, 50)
        dense_bytes = base.B * base.Hkv * base.S * 2 * base.D * base.elem_bytes
        for d in sorted({w.d for w in variants}):
            lay = api.make_layout(base.B, base.Hq, base.Hkv, base.D, d, base.S, tdt)
            klos = [kf[..., :d].contiguous() for kf in kfs]
            khis = [kf[..., d:].contiguous() if d < base.D else None for kf in kfs]
            for w in [w for w in variants if w.d == d]:
                for mode in modes:
                    # a workspace allocated once, cleared, and written by the library alone, as a
                    # serving loop holds it: the launch with cooperating blocks per unit (few
                    # units, long sequences) then needs no clearing kernel in front
                    ws = api.alloc_workspace(lay, w.S, w.d, w.k, mode, zeroed=True)
                    mode_ws = mode | api.WORKSPACE_ZEROED

                    def loki_step(i):
                        c = i % copies
                        api.loki_decode_attn(lay, q, P, klos[c], khis[c], vs[c], w.S, w.d, w.k, mode_ws, ws,
                                             out, None, stream)

                    l_us, l_wall = event_timed_steps(torch, loki_step, steps, 10, stream)
                    kern = kernel_times(api, loki_step, 30)
                    med = _pct(l_us, 50)
                    ab = algorithmic_bytes(w, mode)
                    grouped_literal = (mode == 0 and w.G > 1)
                    e = {"workload": name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "S": w.S, "d": w.d,
                         "k": w.k, "select_mode": mode, "units": w.B * w.Hkv, "steps": steps,
                         "cache_copies": copies, "workspace": "zeroed once, then the library's alone",
                         "us_per_step": med, "us_p10": _pct(l_us, 10), "us_p90": _pct(l_us, 90),
                         "us_mean": float(np.mean(l_us)), "us_wall_clock": l_wall,
                         "tokens_heads_per_s": w.B * w.Hq / (med * 1e-6),
                         "dense_us_per_step": dense_us, "dense_us_p10": _pct(d_us, 10),
                         "dense_us_p90": _pct(d_us, 90),
                         "dense_hbm_gbps": dense_bytes / dense_us / 1e3,
                         "speedup_vs_dense": dense_us / med,
                         "kernels_us": kern,
                         "dominant_kernel": max(kern, key=lambda n: kern[n]) if kern else None}
                    if w.G > 1 and mode == 1:
                        # the whole step of a grouped-query model: the current token's key and
                        # value appended by the same launches (loki_decode_step)
                        kn = torch.randn((w.B, w.Hkv, w.D), device="cuda").to(tdt)
                        vn = torch.randn((w.B, w.Hkv, w.D), device="cuda").to(tdt)

                        def append_step(i):
                            c = i % copies
                            api.loki_decode_step(lay, q, P, klos[c], khis[c], vs[c], w.S, w.d, w.k, mode_ws,
                                                 ws, out, None, k_new=kn, v_new=vn, stream=stream)

                        a_us, _ = event_timed_steps(torch, append_step, steps, 10, stream)
                        e["step_with_append_us"] = _pct(a_us, 50)
                    # recorded counters (all kernels of one step summed), where the table has the point
                    e["traffic"], e["traffic_recorded_in"] = recorded_traffic(
                        f"{name} d={w.d} k={w.k} mode={mode}", "step")
                    if grouped_literal:
                        # every query head gathers its own k rows; heads of a group pick largely the
                        # same rows and share them in cache, so this is a count of requested bytes,
                        # not of bytes moved, and no fraction of the HBM peak is derived from it
                        e.update({"requested_bytes": ab["step"],
                                  "requested_gbps": ab["step"] / med / 1e3,
                                  "algorithmic_bytes": None, "hbm_gbps": None, "frac_of_peak": None})
                    else:
                        e.update({"algorithmic_bytes": ab["step"], "hbm_gbps": ab["step"] / med / 1e3,
                                  "frac_of_peak": ab["step"] / med / 1e3 / HBM_PEAK_GBPS})
                    entries.append(e)
                    log(f"[bench] {w.name} d={w.d} k={w.k} mode {mode}: {med:.1f} us "
                        f"(p10 {e['us_p10']:.1f}, p90 {e['us_p90']:.1f}), dense {dense_us:.1f} us, "
                        f"frac {e['frac_of_peak']}, kernels {kern}")
                    del ws
            del klos, khis
        del kh, vv, kfs, vs, q, P, out, wsd
        torch.cuda.empty_cache()
    return entries


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="llama2_7b")
    ap.add_argument("--select-mode", type=int, default=0)
    ap.add_argument("--copies", type=int, default=4, help="KV-cache copies cycled through")
    ap.add_argument("--d", type=int, default=None)
    ap.add_argument("--k", type=int, default=None)
    ap.add_argument("--path", choices=["auto", "split", "fused", "cluster"], default="auto",
                    help="kernel sequence: the library's choice, or pinned")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-rotate", action="store_true", help="skip the loki_rotate_keys timing")
    ap.add_argument("--no-variants", action="store_true",
                    help="skip Exact-TopK (d = D) and PCAAttn (Algorithm 2) on the same shape")
    ap.add_argument("--no-pca-fit", action="store_true",
                    help="skip the calibration timing (loki_pca_fit on synthetic keys)")
    ap.add_argument("--no-step", action="store_true",
                    help="skip the loki_decode_step timings (append folded in; ragged batch)")
    ap.add_argument("--configs", choices=["all", "none"], default=None,
                    help="the other four workloads (both select modes, the nine (d, k) points of "
                         "the large-model sweep) in the `configs` array of the JSON line; default: "
                         "all when --workload is the benchmark workload, none otherwise")
    ap.add_argument("--config-steps", type=int, default=200,
                    help="event-timed steps per entry of the `configs` array")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy 5 times (reference point for "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the path needs no collective; "
              "it shards by (batch, KV head)); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2406_02542_amd import api, synth

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    api.lib()  # fail loudly if the HIP library is not built

    cfgs = synth.paper_configs()
    if args.workload not in cfgs:
        raise SystemExit(f"unknown workload {args.workload}; choose from {sorted(cfgs)}")
    w = cfgs[args.workload]
    if args.d is not None:
        w = w.replace(d=args.d)
    if args.k is not None:
        w = w.replace(k=args.k)
    mode = args.select_mode
    # the workspace is allocated once, cleared, and written by the library alone (see `ws` below)
    path_bits = {"auto": 0, "split": api.PATH_SPLIT, "fused": api.PATH_FUSED,
                 "cluster": api.PATH_CLUSTER}[args.path] | api.WORKSPACE_ZEROED
    tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16

    log(f"[bench] generating {w}")
    t0 = time.perf_counter()
    x = synth.make_inputs(w, threads=min(16, os.cpu_count() or 8))
    log(f"[bench] inputs in {time.perf_counter() - t0:.1f} s; uploading {args.copies} cache copies")

    lay = api.make_layout(w.B, w.Hq, w.Hkv, w.D, w.d, w.S, tdt)
    kh = torch.from_numpy(x["khat"]).to("cuda").to(tdt)
    vv = torch.from_numpy(x["v"]).to("cuda").to(tdt)
    caches = []
    for _ in range(args.copies):
        klo = kh[..., :w.d].contiguous()
        khi = kh[..., w.d:].contiguous() if w.d < w.D else None
        caches.append((klo, khi, vv.clone(), kh.clone()))
    del kh, vv
    q = torch.from_numpy(x["q"]).to("cuda").to(tdt)
    P = torch.from_numpy(x["P"]).to("cuda")
    ws = api.alloc_workspace(lay, w.S, w.d, w.k, mode, zeroed=True)
    wsd = torch.empty(max(api.loki_workspace_bytes(lay, w.S, 0, 0, -1), 256), dtype=torch.uint8,
                      device="cuda")
    out = torch.empty((w.B, w.Hq, w.D), dtype=tdt, device="cuda")
    stream = torch.cuda.current_stream()

    def loki_step(i):
        klo, khi, v, _ = caches[i % len(caches)]
        api.loki_decode_attn(lay, q, P, klo, khi, v, w.S, w.d, w.k, mode | path_bits, ws, out, None,
                             stream)

    def dense_step(i):
        _, _, v, kf = caches[i % len(caches)]
        api.dense_decode_attn(lay, q, kf, v, w.S, wsd, out, stream)

    def timed(step_fn, steps, warmup):
        # untimed: at least `warmup` steps and at least ~50 ms of work, so that clocks have
        # settled before the timed region starts
        t_w = time.perf_counter()
        i = 0
        while i < warmup or time.perf_counter() - t_w < 0.05:
            step_fn(i)
            i += 1
            if i % 50 == 0:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in range(steps):
            step_fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / steps

    def per_kernel(step_fn, steps):
        prof = api.Profile()
        acc, order = {}, []
        prof.attach()
        try:
            for i in range(steps):
                step_fn(i)
                for name, ms in prof.read():
                    if name not in acc:
                        acc[name] = []
                        order.append(name)
                    acc[name].append(ms)
        finally:
            api.Profile.detach()
            prof.close()
        return {n: float(np.mean(acc[n])) * 1e3 for n in order}  # microseconds

    if args.calibrate_copy:
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    log("[bench] timing loki")
    t_loki = timed(loki_step, args.steps, args.warmup)
    log(f"[bench] loki {t_loki * 1e6:.1f} us/step; per-kernel pass")
    # distribution of step times: each step from one event on the launch stream to the next
    dist_us, _ = event_timed_steps(torch, loki_step, max(200, args.steps), args.warmup, stream)
    step_dist = {"steps": len(dist_us), "median_us": _pct(dist_us, 50), "p10_us": _pct(dist_us, 10),
                 "p90_us": _pct(dist_us, 90), "mean_us": float(np.mean(dist_us)),
                 "std_over_mean": float(np.std(dist_us) / np.mean(dist_us))}

    # the same steps replayed from a captured graph (one step per cache copy in the graph): the
    # library allocates nothing and records no memset, so its launches can be captured as they are
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        graph.capture_begin()
        for i in range(len(caches)):
            klo_, khi_, v_, _ = caches[i]
            api.loki_decode_attn(lay, q, P, klo_, khi_, v_, w.S, w.d, w.k, mode | path_bits, ws, out,
                                 None, side)
        graph.capture_end()
    torch.cuda.synchronize()
    n_rep = max(1, args.steps // len(caches))
    for _ in range(3):
        graph.replay()
    torch.cuda.synchronize()
    t_g = time.perf_counter()
    for _ in range(n_rep):
        graph.replay()
    torch.cuda.synchronize()
    t_graph = (time.perf_counter() - t_g) / (n_rep * len(caches))
    log(f"[bench] loki from a captured graph {t_graph * 1e6:.1f} us/step")
    k_loki = per_kernel(loki_step, args.steps)
    t_dense, k_dense = None, {}
    if not args.no_dense:
        log("[bench] timing dense baseline")
        t_dense = timed(dense_step, args.steps, args.warmup)
        k_dense = per_kernel(dense_step, args.steps)
        log(f"[bench] dense {t_dense * 1e6:.1f} us/step")

    # key rotation + append (Algorithm 1 lines 3-4): whole-prompt prefill and one-token append
    rot = None
    if not args.no_rotate:
        log("[bench] timing loki_rotate_keys")
        gen = torch.Generator(device="cuda")
        gen.manual_seed(w.seed)
        k_pre = torch.randn((w.B, w.Hkv, w.S, w.D), device="cuda", generator=gen).to(tdt)
        k_one = k_pre[:, :, :1, :].contiguous()
        rklo, rkhi, _ = api.alloc_cache(lay)

        def rot_prefill(i):
            api.loki_rotate_keys(lay, k_pre, P, rklo, rkhi, 0, w.S, stream)

        def rot_append(i):
            api.loki_rotate_keys(lay, k_one, P, rklo, rkhi, w.S - 1, 1, stream)

        t_pre = timed(rot_prefill, max(10, args.steps // 10), 3)
        t_app = timed(rot_append, args.steps, args.warmup)
        pre_bytes = 2 * w.B * w.Hkv * w.S * w.D * w.elem_bytes  # read K, write Khat
        rot = {"prefill_us": t_pre * 1e6, "prefill_rows": w.B * w.Hkv * w.S,
               "prefill_hbm_gbps": pre_bytes / t_pre / 1e9,
               "prefill_hbm_frac": pre_bytes / t_pre / 1e9 / HBM_PEAK_GBPS,
               "append_one_token_us": t_app * 1e6}
        log(f"[bench] rotate prefill {t_pre * 1e6:.1f} us, append {t_app * 1e6:.1f} us")
        del k_pre, k_one, rklo, rkhi

    # the whole step with the cache append folded in, and a ragged batch (loki_decode_step)
    step = None
    if not args.no_step:
        log("[bench] timing loki_decode_step")
        st_in = synth.make_step_inputs(w, x["P"], ragged=True)
        k_new = torch.from_numpy(st_in["k_new"]).to("cuda").to(tdt)
        v_new = torch.from_numpy(st_in["v_new"]).to("cuda").to(tdt)
        lens = torch.from_numpy(st_in["seq_lens"]).to("cuda")
        ks = torch.from_numpy(st_in["ks"]).to("cuda")

        def append_step(i):
            klo, khi, v, _ = caches[i % len(caches)]
            api.loki_decode_step(lay, q, P, klo, khi, v, w.S, w.d, w.k, mode | path_bits, ws, out,
                                 None, k_new=k_new, v_new=v_new, stream=stream)

        def separate_step(i):
            klo, khi, v, _ = caches[i % len(caches)]
            api.loki_rotate_keys(lay, k_new.view(w.B, w.Hkv, 1, w.D), P, klo, khi, w.S - 1, 1, stream)
            v[:, :, w.S - 1, :] = v_new
            api.loki_decode_attn(lay, q, P, klo, khi, v, w.S, w.d, w.k, mode | path_bits, ws, out,
                                 None, stream)

        def ragged_step(i):
            klo, khi, v, _ = caches[i % len(caches)]
            api.loki_decode_step(lay, q, P, klo, khi, v, w.S, w.d, w.k, mode | path_bits, ws, out,
                                 None, seq_lens=lens, ks=ks, k_new=k_new, v_new=v_new, stream=stream)

        def ragged_dense(i):
            _, _, v, kf = caches[i % len(caches)]
            api.dense_decode_step(lay, q, kf, v, w.S, lens, wsd, out, stream)

        # the same step on a paged cache: the rows of cache copy 0 scattered over randomly ordered
        # physical pages of 256 rows (a quarter of the pool unused)
        page_rows = 256
        pps = (w.S + page_rows - 1) // page_rows
        n_pages = w.B * pps * 4 // 3 + 1
        gen_p = torch.Generator(device="cpu")
        gen_p.manual_seed(w.seed)
        table = torch.randperm(n_pages, generator=gen_p)[:w.B * pps].to(torch.int32).view(w.B, pps).cuda()

        def to_pool(c):
            pool = torch.zeros((n_pages, w.Hkv, page_rows, c.shape[-1]), dtype=tdt, device="cuda")
            pad = pps * page_rows - c.shape[2]
            if pad:
                c = torch.nn.functional.pad(c, (0, 0, 0, pad))
            pool[table.view(-1).long()] = c.view(w.B, w.Hkv, pps, page_rows, -1).permute(0, 2, 1, 3, 4).reshape(
                w.B * pps, w.Hkv, page_rows, -1)
            return pool

        pools = [to_pool(caches[0][0]), to_pool(caches[0][1]) if caches[0][1] is not None else None,
                 to_pool(caches[0][2])]

        def paged_step(i):
            api.loki_decode_step(lay, q, P, pools[0], pools[1], pools[2], w.S, w.d, w.k, mode | path_bits,
                                 ws, out, None, k_new=k_new, v_new=v_new, page_table=table,
                                 page_rows=page_rows, n_pages=n_pages, stream=stream)

        t_paged = timed(paged_step, args.steps, args.warmup)
        del pools

        # several new tokens per sequence (chunked / speculative decoding): the same number of
        # batch entries, as m = 4 consecutive tokens of B / 4 sequences (the first B / 4 caches)
        multi = None
        m_tok = 4
        if w.B % m_tok == 0 and w.B * w.Hq * 1 <= 65535:
            bs = w.B // m_tok
            lay_m = api.make_layout(bs, w.Hq, w.Hkv, w.D, w.d, caches[0][0].shape[2], tdt)
            lens_m = torch.tensor([w.S - (m_tok - 1 - j) for _ in range(bs) for j in range(m_tok)],
                                  dtype=torch.int32, device="cuda")
            ks_m = torch.full((w.B,), w.k, dtype=torch.int32, device="cuda")

            def multi_step(i):
                klo, khi, v, _ = caches[i % len(caches)]
                api.loki_decode_step(lay_m, q, P, klo, khi, v, w.S, w.d, w.k, mode, ws, out, None,
                                     seq_lens=lens_m, ks=ks_m, k_new=k_new, v_new=v_new,
                                     queries_per_seq=m_tok, stream=stream)

            t_multi = timed(multi_step, args.steps, args.warmup)
            multi = {"queries_per_seq": m_tok, "sequences": bs, "us": t_multi * 1e6,
                     "us_per_token": t_multi * 1e6 / m_tok}
            log(f"[bench] {m_tok} tokens per sequence on {bs} sequences: {t_multi * 1e6:.1f} us")
        t_app = timed(append_step, args.steps, args.warmup)
        t_sep = timed(separate_step, args.steps, args.warmup)
        t_rag = timed(ragged_step, args.steps, args.warmup)
        t_rd = timed(ragged_dense, args.steps, args.warmup)
        e = w.elem_bytes
        sel_per_unit = 1 if (mode == 1 or w.G == 1) else w.G
        rag_bytes = float(sum(w.Hkv * (int(L) * w.d + sel_per_unit * int(K) * 2 * w.D) * e
                              for L, K in zip(st_in["seq_lens"], st_in["ks"])))
        rag_dense_bytes = float(sum(w.Hkv * int(L) * 2 * w.D * e for L in st_in["seq_lens"]))
        step = {"append_folded_in_us": t_app * 1e6,
                "paged_cache": {"page_rows": page_rows, "pool_pages": n_pages,
                                "append_folded_in_us": t_paged * 1e6},
                "rotate_keys_then_value_copy_then_decode_us": t_sep * 1e6,
                "several_tokens_per_sequence": multi,
                "ragged": {"seq_lens_min_mean_max": [int(st_in["seq_lens"].min()),
                                                     float(st_in["seq_lens"].mean()),
                                                     int(st_in["seq_lens"].max())],
                           "us": t_rag * 1e6, "hbm_gbps": rag_bytes / t_rag / 1e9,
                           "dense_us": t_rd * 1e6, "dense_hbm_gbps": rag_dense_bytes / t_rd / 1e9,
                           "speedup_vs_dense": t_rd / t_rag}}
        log(f"[bench] paged cache, step with append {t_paged * 1e6:.1f} us")
        log(f"[bench] step with append {t_app * 1e6:.1f} us (separate calls {t_sep * 1e6:.1f} us); "
            f"ragged {t_rag * 1e6:.1f} us, dense ragged {t_rd * 1e6:.1f} us")

    # the paper's two comparison variants on the same kernels: Exact-TopK (Section 5: d = D, the
    # ranking scores are the exact logits) and PCAAttn (Appendix E, Algorithm 2)
    variants = None
    if not args.no_variants:
        log("[bench] timing Exact-TopK and PCAAttn")
        e = w.elem_bytes
        units = w.B * w.Hkv
        sel_per_unit = 1 if (mode == 1 or w.G == 1) else w.G
        lay_full = api.make_layout(w.B, w.Hq, w.Hkv, w.D, w.D, w.S, tdt)
        ws_full = api.alloc_workspace(lay_full, w.S, w.D, w.k, mode)
        ws_pca = torch.empty(api.loki_workspace_bytes(lay, w.S, w.d, 0, -2), dtype=torch.uint8,
                             device="cuda")

        def exact_topk_step(i):
            _, _, v, kf = caches[i % len(caches)]  # the unsplit rotated cache is the d = D layout
            api.loki_decode_attn(lay_full, q, P, kf, None, v, w.S, w.D, w.k, mode, ws_full, out, None,
                                 stream)

        def pca_step(i):
            klo, _, v, _ = caches[i % len(caches)]
            api.loki_pca_attn(lay, q, P, klo, v, w.S, w.d, ws_pca, out, stream)

        t_et = timed(exact_topk_step, args.steps, args.warmup)
        t_pca = timed(pca_step, args.steps, args.warmup)
        # Exact-TopK: S D for the scores; with one query head per KV head the scores are the logits
        # and only the k value rows follow, otherwise k key and value rows per selecting head
        row_elems = w.D if w.G == 1 else 2 * w.D
        et_bytes = units * (w.S * w.D + sel_per_unit * w.k * row_elems) * e
        pca_bytes = units * w.S * (w.d + w.D) * e
        variants = {"exact_topk": {"d": w.D, "k": w.k, "us": t_et * 1e6, "algorithmic_bytes": et_bytes,
                                   "hbm_gbps": et_bytes / t_et / 1e9},
                    "pca_attn": {"d": w.d, "us": t_pca * 1e6, "algorithmic_bytes": pca_bytes,
                                 "hbm_gbps": pca_bytes / t_pca / 1e9}}
        log(f"[bench] Exact-TopK {t_et * 1e6:.1f} us, PCAAttn {t_pca * 1e6:.1f} us")
        del ws_full, ws_pca

    # calibration (Section 3.1): PCA of 65 536 keys per KV head of the workload's shape
    pca = None
    if not args.no_pca_fit:
        log("[bench] timing loki_pca_fit")
        n_cal = 65536
        gen = torch.Generator(device="cuda")
        gen.manual_seed(w.seed + 1)
        cal = torch.randn((w.Hkv, n_cal, w.D), device="cuda", generator=gen).to(tdt)
        Pfit = torch.empty((w.Hkv, w.D, w.D), device="cuda")
        lam = torch.empty((w.Hkv, w.D), device="cuda")
        wsp = torch.empty(api.loki_pca_workspace_bytes(lay, n_cal), dtype=torch.uint8, device="cuda")

        def fit_step(i):
            api.loki_pca_fit(lay, cal, n_cal, Pfit, lam, wsp, stream)

        t_fit = timed(fit_step, 5, 1)
        k_fit = per_kernel(fit_step, 5)
        gram_bytes = w.Hkv * n_cal * w.D * w.elem_bytes
        pca = {"keys_per_head": n_cal, "heads": w.Hkv, "us": t_fit * 1e6, "stages_us": k_fit,
               "gram_hbm_gbps": gram_bytes / (k_fit["pca_gram"] * 1e-6) / 1e9}
        log(f"[bench] pca_fit {t_fit * 1e6:.0f} us: {k_fit}")
        del cal, wsp

    ab = algorithmic_bytes(w, mode)

    # the read ceiling of this device: a trivial kernel streaming as many bytes as one decode
    # step moves (algorithmic bytes), over buffers cycled like the cache copies
    step_bytes = int(ab["step"]) // 16 * 16
    sbufs = [torch.empty(step_bytes, dtype=torch.uint8, device="cuda").random_(0, 255)
             for _ in range(max(3, args.copies))]
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(10):
        api.loki_stream_read(sbufs[i % len(sbufs)], step_bytes, stream)
    n_sr = max(20, args.steps // 4)
    ev0.record(stream)
    for i in range(n_sr):
        api.loki_stream_read(sbufs[i % len(sbufs)], step_bytes, stream)
    ev1.record(stream)
    torch.cuda.synchronize()
    sr_us = ev0.elapsed_time(ev1) * 1e3 / n_sr
    del sbufs
    stream_read = {"bytes": step_bytes, "us": sr_us, "GB/s": step_bytes / sr_us / 1e3,
                   "frac_of_peak": step_bytes / sr_us / 1e3 / HBM_PEAK_GBPS}
    log(f"[bench] plain read of {step_bytes} bytes: {sr_us:.1f} us")

    # the longest kernel of the step, whether or not the method assigns it bytes (select, query
    # rotation and merge kernels move none: their time is overhead on the step's roofline)
    dominant = max(k_loki, key=lambda n: k_loki[n])
    kernel_us = k_loki[dominant]
    if len(k_loki) == 1:
        # The step is this one kernel: its average launch duration is the span between two
        # events on the launch stream around the timed launches, divided by their number (the
        # same way the plain read above is timed).  The per-launch events of the profile hook
        # are each read back before the next launch, so there every launch starts on an idle
        # device and the event pair itself adds to the span; that figure stays as
        # kernel_us_isolated.
        for i in range(max(args.warmup, 20)):
            loki_step(i)
        ev0.record(stream)
        for i in range(args.steps):
            loki_step(i)
        ev1.record(stream)
        torch.cuda.synchronize()
        kernel_us = ev0.elapsed_time(ev1) * 1e3 / args.steps
        log(f"[bench] {dominant}: {kernel_us:.1f} us per launch between events "
            f"({k_loki[dominant]:.1f} us isolated)")
    dom_bytes = ab.get(dominant, 0)
    achieved = dom_bytes / (kernel_us * 1e-6) / 1e9
    default_shape = (w == cfgs[args.workload]) and mode == 0
    traffic, traffic_source = recorded_traffic(w.name, dominant) if default_shape else (None, None)
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                "traffic_recorded_in": traffic_source,
                "algorithmic_bytes": dom_bytes, "kernel_us": kernel_us,
                "kernel_us_isolated": k_loki[dominant],
                "stream_read": stream_read,
                "frac_of_stream_read": achieved / stream_read["GB/s"]}

    result = {
        "metric": "loki_decode_attn_us_per_step",
        "value": t_loki * 1e6,
        "unit": "us/step",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": t_loki * 1e3,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D, "S": w.S,
                   "d": w.d, "k": w.k, "select_mode": mode, "path": args.path, "cache_copies": args.copies},
        "tokens_heads_per_s": w.B * w.Hq / t_loki,
        "step_hbm_gbps": ab["step"] / t_loki / 1e9,
        "step_hbm_frac": ab["step"] / t_loki / 1e9 / HBM_PEAK_GBPS,
        "step_time_distribution": step_dist,
        "graph_replay_us_per_step": t_graph * 1e6,
        "kernels_us": k_loki,
        "dense_us_per_step": t_dense * 1e6 if t_dense else None,
        "dense_hbm_gbps": ab["dense_attend"] / t_dense / 1e9 if t_dense else None,
        "dense_kernels_us": k_dense,
        "speedup_vs_dense": (t_dense / t_loki) if t_dense else None,
        "rotate_keys": rot,
        "decode_step": step,
        "variants": variants,
        "pca_fit": pca,
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle on a sample")
        result["cpu_baseline"] = cpu_baseline(w, x, mode)
    else:
        result["cpu_baseline"] = None
    want_configs = args.configs or ("all" if (args.workload == "llama2_7b" and default_shape) else "none")
    if want_configs == "all":
        # free the benchmark workload's tensors first: the other workloads hold up to 2 GiB caches
        del caches, x
        torch.cuda.empty_cache()
        result["configs"] = bench_configs(args, torch, api, synth)
    else:
        result["configs"] = None
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
