#!/usr/bin/env python3
"""Benchmark of the LineAR decode path on one MI355X.

A *step* is one decode step of the whole workload: decode_step for every layer (append +
attention + guide-queue append), plus, when the step closes a raster line, end_of_line_evict
for every layer (saliency, selection, compaction).  All inputs are resident in HBM before any
timed region starts.

Two things are timed for the compressed cache and, over the same step indices, for the same
kernels on the full cache (B = N):
  * the K-step window (`--steps K`): K consecutive steps of an image in the steady state of
    the method -- behind the first eviction, ending with the end-of-line call of an evicting
    line -- reached by running the image's earlier steps untimed (the last `--warmup` of them
    are the warm-up).  `value` is this window's time per step;
  * one whole image (all N steps from the first token), whatever K is: whole-image time, the
    first-half / last-half means (the paper's Fig. 8 view) and the whole-image speed-up.
The same whole-image pair is measured for each of the four benchmark workloads
(`per_workload`).  One JSON line goes to stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published peak
PAPER_CONTEXT = {          # end-to-end speedups the paper prints (Table 4 / Table 1), NVIDIA A800
    "llamagen-xl": 7.57, "janus-pro-7b": 5.62, "janus-pro-1b": 5.87, "lumina-mgpt-768": 2.13}
TABLE_WORKLOADS = ("llamagen-xl", "janus-pro-1b", "janus-pro-7b", "lumina-mgpt-768")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


# ------------------------------------------------------------------ host-side accounting ---
def visual_len_at(w, step):
    """Visual tokens in the cache when 0-based decode step `step` attends (its own included):
    grows to B, then saw-tooths between B-n+1 and B (Sec. 3.3: B - n retained after each
    eviction plus the line being written)."""
    n, B = w.line_len, w.budget
    i = step + 1
    return i if i <= B else B - n + ((i - 1) % n) + 1


def sum_keys(w, steps, start=0):
    """Keys read per pair over decode steps [start, start + steps)."""
    return sum(w.n_cond + visual_len_at(w, s) for s in range(start, start + steps))


def evicting_line(w, line):
    """Does the end of 1-based raster line `line` evict?  Lines B/n .. h-1 do (Sec. 3.3)."""
    return w.budget < w.n_visual and w.budget // w.line_len <= line <= w.n_lines - 1


def evicting_ends_in(w, start, steps):
    """Evicting end-of-line calls inside the window of decode steps [start, start + steps): the
    call that follows step index l*n - 1 belongs to the window that contains that step."""
    n = w.line_len
    return [l for l in range(1, w.n_lines + 1) if start < l * n <= start + steps and evicting_line(w, l)]


def steady_window(w, steps):
    """(start, steps) of the timed window: `steps` consecutive decode steps that end with the
    end-of-line call of an evicting line and, when the image is long enough, start behind the
    first eviction.  A whole image (steps >= N) starts at its first token."""
    n, h, N = w.line_len, w.n_lines, w.n_visual
    steps = max(1, min(steps, N))
    if w.budget >= N or steps >= N:
        return 0, steps
    first = w.budget // n                                  # first evicting line (1-based), <= h - 1
    last_line = min(h - 1, first + math.ceil(steps / n))   # the window ends with this line's eviction
    start = max(0, last_line * n - steps)
    # never a window in which the two legs do the same work: extend it until it holds an evicting
    # end of line and the compressed leg reads fewer keys than the full-cache leg
    while steps < N and (not evicting_ends_in(w, start, steps) or
                         sum_keys(w, steps, start) >= sum_keys(w.full_cache(), steps, start)):
        steps = min(N, steps + n)
        start = max(0, min(start, N - steps))
    return start, steps


# ------------------------------------------------------------------------ CPU oracle leg ---
def _oracle_worker(args):
    """One process: whole-image replays of single (layer, sequence, head) slices until the
    deadline; returns (replays, seconds spent in them)."""
    name, overrides, head0, n_heads, deadline, max_replays = args
    import importlib.util

    import torch
    from threadpoolctl import threadpool_limits

    from paper_2512_04857_amd import synth
    from dataclasses import replace

    torch.set_num_threads(1)
    w = replace(synth.WORKLOADS[name], **overrides)
    spec = importlib.util.spec_from_file_location("linear_oracle", os.path.join(ROOT, "oracle", "linear_oracle.py"))
    o = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(o)
    ws = synth.shrink(w, n_layers=1, batch=1, n_heads=n_heads)
    kc, vc = synth.cond_kv(ws)
    q, k, v = synth.image_qkv(ws)
    f = lambda t: t.to(torch.float64).numpy()
    kc, vc, q, k, v = f(kc[0, 0]), f(vc[0, 0]), f(q[:, 0, 0]), f(k[:, 0, 0]), f(v[:, 0, 0])
    done, spent = 0, 0.0
    with threadpool_limits(limits=1):
        while done < max_replays and (done == 0 or time.time() < deadline):
            hd = (head0 + done) % n_heads
            t0 = time.perf_counter()
            o.run_slice(kc[hd], vc[hd], q[:, hd], k[:, hd], v[:, hd], line_len=w.line_len, n_lines=w.n_lines,
                        budget=w.budget, n_init=w.n_init, n_recent_lines=w.n_recent_lines)
            spent += time.perf_counter() - t0
            done += 1
    return done, spent


def cpu_baseline(w, base_name, overrides, budget_s: float):
    """The CPU oracle as it stands on the host's cores: one process per core, each replaying
    whole images of single slices of the workload (slices are independent, so the whole
    workload costs slices x this) for about `budget_s` seconds.  `w` is synth.WORKLOADS[base_name]
    with `overrides` applied.  Runs before the GPU is touched."""
    import multiprocessing as mp

    try:
        avail = len(os.sched_getaffinity(0))
    except AttributeError:
        avail = os.cpu_count() or 1
    cores = max(1, min(avail, 16))          # a one-GPU machine grants 16 cores whatever it reports
    n_heads = min(w.n_heads, 8)
    t0 = time.time()
    deadline = t0 + budget_s
    jobs = [(base_name, overrides, i, n_heads, deadline, 10 ** 6) for i in range(cores)]
    with mp.get_context("fork").Pool(cores) as pool:
        res = pool.map(_oracle_worker, jobs)
    wall = time.time() - t0
    done = sum(r[0] for r in res)
    spent = sum(r[1] for r in res)
    total_slices = w.n_layers * w.batch * w.n_heads
    one = spent / done / w.n_visual * total_slices * 1e6          # one core doing everything
    return {"value": round(one / cores, 1), "unit": "us/step", "cores": cores, "kind": "oracle",
            "cores_visible": avail, "single_core_us_per_step": round(one, 1),
            "sample": f"{done} whole-image replays ({w.n_visual} steps each) of single (layer, sequence, head) "
                      f"slices on {cores} processes in {wall:.1f} s ({spent:.1f} core-seconds in the replays), "
                      f"scaled linearly to the workload's {total_slices} slices and divided by the cores"}


# ------------------------------------------------------------------------------ GPU legs ---
class Runner:
    """Pre-generated inputs and raw-pointer launch loops for one workload."""

    def __init__(self, w, device):
        import torch

        from paper_2512_04857_amd import binding, synth

        self.torch, self.binding, self.w, self.device = torch, binding, w, device
        t0 = time.perf_counter()
        self.kc, self.vc = synth.cond_kv(w, device)
        self.q, self.k, self.v = synth.image_qkv(w, device)          # [N, L, Bz, H, d]
        torch.cuda.synchronize()
        log(f"inputs for {w.name}: {3 * self.q.numel() * self.q.element_size() / 1e9:.2f} GB generated in "
            f"{time.perf_counter() - t0:.1f} s")
        self.out = torch.empty((w.n_layers, w.batch, w.n_heads, w.head_dim), dtype=torch.float32, device=device)
        self.stride = self.q[0, 0].numel() * self.q.element_size()
        self.ostride = self.out[0].numel() * 4
        self.table = None

    def run(self, wl, start, steps, warmup, groups_per_wave=0, n_split=0, score_mode=0, guide_queue=0,
            fused_rope=False):
        """Times decode steps [start, start + steps) of an image of workload variant `wl` (same
        shapes, its own budget), end-of-line calls included; steps [0, start) run untimed first
        (when start < warmup a throw-away image of `warmup` steps runs before).  Returns a dict
        of measurements."""
        torch, binding = self.torch, self.binding
        L, n, N = wl.n_layers, wl.line_len, wl.n_visual
        cache = binding.LineARCache(binding.cfg_from_workload(wl, score_mode=score_mode, guide_queue=guide_queue),
                                    self.device)
        lib = binding.lib()
        dsteps, evicts = lib.decode_step_layers, lib.end_of_line_evict_layers
        if fused_rope:
            # the rotary embedding fused into the step: the pre-generated q, k stand in for unrotated
            # ones (the timing does not depend on the values); one table row per position
            from paper_2512_04857_amd import synth
            if self.table is None:
                self.table = torch.stack([synth.rope_cos_sin(wl, wl.n_cond + i, self.device) for i in range(N)])
            tb, tst = self.table.data_ptr(), self.table[0].numel() * 4
            rope = lib.decode_step_rope_layers
        qb, kb, vb, ob = self.q.data_ptr(), self.k.data_ptr(), self.v.data_ptr(), self.out.data_ptr()
        st, ost = self.stride, self.ostride
        stream = cache.stream()

        def begin():
            cache.start_image(self.kc, self.vc)
            if groups_per_wave or n_split:
                binding.linear_set_tuning(cache.handle, groups_per_wave, n_split)

        def play(s_from, s_to, events):
            h = cache.handle
            mark = (lambda kind: None) if events is None else (lambda kind: events.append((kind, self._event())))
            mark("start")
            for s in range(s_from, s_to):
                off = s * L * st
                if fused_rope:
                    rc = rope(h, 0, L, qb + off, kb + off, vb + off, tb + s * tst, ob, st, ost, stream)
                else:
                    rc = dsteps(h, 0, L, qb + off, kb + off, vb + off, ob, st, ost, stream)
                if rc:
                    raise binding.LinearError(rc, "decode_step_layers")
                if (s + 1) % n == 0:
                    mark("decode_end")
                    rc = evicts(h, 0, L, stream)
                    if rc:
                        raise binding.LinearError(rc, "end_of_line_evict_layers")
                    mark("line_end")
            mark("stop")

        if start < warmup:
            begin()
            play(0, min(warmup, N), None)
        begin()
        play(0, start, None)
        torch.cuda.synchronize()
        ev = []
        t0 = time.perf_counter()
        play(start, start + steps, ev)
        enqueue = time.perf_counter() - t0
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        cache.close()

        total_ms = ev[0][1].elapsed_time(ev[-1][1])
        # split the timeline into decode spans and eviction spans, line by line
        decode_ms, evict_ms, line_ms = 0.0, 0.0, []
        prev = ev[0][1]
        for kind, e in ev[1:]:
            dt = prev.elapsed_time(e)
            if kind == "decode_end":
                decode_ms += dt
                line_ms.append(dt)
            elif kind == "line_end":
                evict_ms += dt
                line_ms[-1] += dt
            else:                      # trailing partial line
                decode_ms += dt
            prev = e
        ev_lines = evicting_ends_in(wl, start, steps)
        keys = sum_keys(wl, steps, start)
        tok_bytes = 2 * wl.n_heads * wl.head_dim * self.q.element_size() * wl.batch
        launches = steps * L
        res = {
            "start_step": start,
            "steps": steps,
            "us_per_step": total_ms * 1e3 / steps,
            "total_ms": total_ms,
            "host_wall_ms": wall * 1e3,
            "host_enqueue_ms": enqueue * 1e3,
            "decode_ms": decode_ms,
            "evict_ms": evict_ms,
            "decode_launches": launches,
            "decode_us_per_launch": decode_ms * 1e3 / launches,
            "evicting_lines": len(ev_lines),
            "evict_us_per_layer": (evict_ms * 1e3 / (len(ev_lines) * L)) if ev_lines else None,
            "kv_bytes_per_launch": keys * tok_bytes / steps,
            "kv_bytes_total": keys * tok_bytes * L,
            "mean_keys": keys / steps,
        }
        res["achieved_GBs"] = res["kv_bytes_per_launch"] / (res["decode_us_per_launch"] * 1e-6) / 1e9
        if start == 0 and steps == N:
            half = wl.n_lines // 2
            res["us_per_step_first_half"] = sum(line_ms[:half]) / (half * n) * 1e3 if half else None
            res["us_per_step_last_half"] = sum(line_ms[wl.n_lines - half:]) / (half * n) * 1e3 if half else None
            res["line_us_per_launch"] = [round(x * 1e3 / (n * L), 2) for x in line_ms]
        return res

    def _event(self):
        e = self.torch.cuda.Event(enable_timing=True)
        e.record()
        return e


def probe(w, device, reps=3):
    """What the decode launches are measured against, on the same cache buffers and launch
    pattern (one launch per layer per token, back to back, all layers cycling): a kernel that
    only reads the K and V rows a decode step reads (no arithmetic, no store), over the whole
    image's cache-length trajectory and at fixed lengths; and an empty kernel."""
    import torch

    from paper_2512_04857_amd import binding

    cfg = binding.cfg_from_workload(w)
    cache = binding.LineARCache(cfg, device)
    for t in cache.k_cache + cache.v_cache:
        t.zero_()
    kp, vp = [t.data_ptr() for t in cache.k_cache], [t.data_ptr() for t in cache.v_cache]
    L, N, P = w.n_layers, w.n_visual, w.batch * w.n_heads
    row_bytes = w.head_dim * cache.k_cache[0].element_size()
    stream = cache.stream()

    def timed(fn):
        best = None
        for _ in range(reps):
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
        return best

    def stream_rows(rows_list):
        def fn():
            for rows in rows_list:
                binding.linear_probe_stream(kp, vp, P, rows, cache.t_max, row_bytes, stream)
        ms = timed(fn)
        launches = len(rows_list) * L
        byts = sum(rows_list) * 2 * P * row_bytes * L
        return {"us_per_launch": round(ms * 1e3 / launches, 3), "GBs": round(byts / ms / 1e6, 1),
                "bytes_per_launch": round(byts / launches), "launches": launches}

    image_rows = [w.n_cond + visual_len_at(w, s) - 1 for s in range(N)]
    image_rows = [max(r, 1) for r in image_rows]
    mean_rows = max(1, round(sum(image_rows) / N))
    out = {
        "workload": w.name,
        "empty_launch_us": round(timed(lambda: binding.linear_probe_empty(20 * L, P, 64, stream)) * 1e3 / (20 * L), 3),
        "stream_whole_image": stream_rows(image_rows),
        "stream_mean_length": dict(rows=mean_rows, **stream_rows([mean_rows] * 48)),
        "stream_max_length": dict(rows=cache.t_max - 1, **stream_rows([cache.t_max - 1] * 48)),
    }
    cache.close()
    return out


def cache_memory(w, score_mode, guide_queue=0):
    """K/V cache and scratch bytes of the compressed and the full-cache handle (Table 4's memory
    column counts the whole model; this is the cache's share of it)."""
    from paper_2512_04857_amd import binding

    def sizes(wl, mode, queue):
        per_layer, scratch = binding.linear_workspace_bytes(
            binding.cfg_from_workload(wl, score_mode=mode, guide_queue=queue))
        return 2 * per_layer * wl.n_layers, scratch

    ck, cs = sizes(w, score_mode, guide_queue)
    fk, fs = sizes(w.full_cache(), 0, 0)
    return {"compressed_kv_bytes": ck, "compressed_scratch_bytes": cs, "full_kv_bytes": fk,
            "full_scratch_bytes": fs, "saving": round(1.0 - (ck + cs) / (fk + fs), 4)}


def whole_image_summary(w, comp, full):
    """The per-workload record: one whole image on the compressed cache and one on the full cache."""
    r = {
        "us_per_step": round(comp["us_per_step"], 2),
        "whole_image_ms": round(comp["total_ms"], 3),
        "us_per_step_first_half": round(comp["us_per_step_first_half"], 2),
        "us_per_step_last_half": round(comp["us_per_step_last_half"], 2),
        "decode_us_per_launch": round(comp["decode_us_per_launch"], 3),
        "decode_launches": comp["decode_launches"],
        "algorithmic_bytes_per_launch": round(comp["kv_bytes_per_launch"]),
        "achieved_GBs": round(comp["achieved_GBs"], 1),
        "frac_of_hbm_peak": round(comp["achieved_GBs"] / HBM_PEAK_GBS, 4),
        "evict_us_per_layer": round(comp["evict_us_per_layer"], 3) if comp["evict_us_per_layer"] else None,
        "evict_share": round(comp["evict_ms"] / comp["total_ms"], 4),
        "paper_end_to_end_speedup_context": PAPER_CONTEXT.get(w.name),
    }
    if full:
        r["full_cache"] = {
            "us_per_step": round(full["us_per_step"], 2),
            "whole_image_ms": round(full["total_ms"], 3),
            "us_per_step_first_half": round(full["us_per_step_first_half"], 2),
            "us_per_step_last_half": round(full["us_per_step_last_half"], 2),
            "decode_us_per_launch": round(full["decode_us_per_launch"], 3),
            "achieved_GBs": round(full["achieved_GBs"], 1),
            "frac_of_hbm_peak": round(full["achieved_GBs"] / HBM_PEAK_GBS, 4),
        }
        r["speedup_vs_full_cache"] = round(full["total_ms"] / comp["total_ms"], 3)
        r["byte_ratio_full_over_compressed"] = round(full["kv_bytes_total"] / comp["kv_bytes_total"], 3)
    return r


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="decode steps of the timed window (default: one whole image)")
    ap.add_argument("--warmup", type=int, default=48)
    ap.add_argument("--workload", default="llamagen-xl")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="0 skips the CPU oracle leg")
    ap.add_argument("--skip-full", action="store_true", help="do not time the full-cache variant")
    ap.add_argument("--no-whole-image", action="store_true",
                    help="time the window only (profiling runs); the printed line then carries no whole-image keys")
    ap.add_argument("--no-table", action="store_true", help="do not measure the other benchmark workloads")
    ap.add_argument("--probe", action="store_true",
                    help="instead of the benchmark line, print what the decode launches are measured against: a "
                         "read-only streaming kernel over the same rows and launch pattern, an empty kernel, and "
                         "the decode path's whole image beside them")
    ap.add_argument("--calibrate-copy-mib", type=int, default=0,
                    help="also run one elementwise read+write pass over this many MiB (a traffic yardstick for "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs)")
    ap.add_argument("--sequences", type=int, default=0,
                    help="override the number of sequences (e.g. 512 = the paper's Table 4 batch of 256 "
                         "with both guidance halves, for the LlamaGen-XL shape)")
    ap.add_argument("--layers", type=int, default=0,
                    help="override the number of layers (a few layers' caches stay in the last-level cache: a "
                         "diagnostic of cache-resident speed, not a benchmark figure)")
    ap.add_argument("--budget-lines", type=int, default=0,
                    help="override the budget B, in raster lines (rho sweeps: 6 of 24 lines = 1/4, ...)")
    ap.add_argument("--score-mode", type=int, default=0,
                    help="0 = Eq. 9 as printed (default), 1 = decode-softmax mass, 2 = accumulated attention, "
                         "3 = random (seeded hash)")
    ap.add_argument("--guide-queue", type=int, default=0,
                    help="0: automatic; 1: the guide queue holds logits; 2: it holds the queries (score mode 0 only)")
    ap.add_argument("--fused-rope", action="store_true",
                    help="time decode_step_rope (rotary embedding of q and k fused into the step)")
    ap.add_argument("--groups-per-wave", type=int, default=0, help="decode kernel tuning (0 = default)")
    ap.add_argument("--n-split", type=int, default=0, help="decode kernel tuning (0 = automatic)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        return 2

    from dataclasses import replace

    from paper_2512_04857_amd import synth

    w = synth.WORKLOADS[args.workload]
    overrides = {}
    if args.sequences:
        overrides["batch"] = args.sequences
        w = replace(w, batch=args.sequences, name=f"{w.name}-seq{args.sequences}")
    if args.layers:
        overrides["n_layers"] = args.layers
        w = replace(w, n_layers=args.layers, name=f"{w.name}-L{args.layers}")
    if args.budget_lines:
        overrides["budget"] = args.budget_lines * w.line_len
        w = replace(w, budget=args.budget_lines * w.line_len, name=f"{w.name}-b{args.budget_lines}")
    if w.budget >= w.n_visual:
        print("bench.py: the workload's budget holds the whole image, so the compressed and the full-cache "
              "leg would be the same work; choose a budget below N", file=sys.stderr)
        return 2
    N = w.n_visual
    requested = args.steps or N
    start, steps = steady_window(w, requested)
    if requested > N:
        log(f"--steps is capped at one image ({N} decode steps)")
    elif steps != requested:
        log(f"window extended from {requested} to {steps} steps so that it holds an evicting end of line")

    cpu = cpu_baseline(w, args.workload, overrides, args.cpu_seconds) if args.cpu_seconds > 0 else None
    if cpu:
        log("cpu oracle:", cpu)

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    device = "cuda:0"
    r = Runner(w, device)
    if args.calibrate_copy_mib:
        src = torch.empty(args.calibrate_copy_mib << 20, dtype=torch.uint8, device=device).random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1, out=dst)      # an elementwise kernel (a plain copy_ may go to the DMA engines)
        torch.cuda.synchronize()
        log(f"calibration pass (uint8 add kernel): {args.calibrate_copy_mib} MiB read + "
            f"{args.calibrate_copy_mib} MiB written")
        del src, dst
    tune = (args.groups_per_wave, args.n_split)
    variant = (args.score_mode, args.guide_queue, args.fused_rope)
    if args.probe:
        res = {"probe": probe(w, device)}
        img = r.run(w, 0, N, args.warmup, *tune, *variant)
        res["decode_whole_image"] = {"us_per_launch": round(img["decode_us_per_launch"], 3),
                                     "GBs": round(img["achieved_GBs"], 1),
                                     "bytes_per_launch": round(img["kv_bytes_per_launch"]),
                                     "launches": img["decode_launches"]}
        if not args.skip_full:
            res["probe_full_cache"] = probe(w.full_cache(), device)
            imgf = r.run(w.full_cache(), 0, N, args.warmup, *tune)
            res["decode_whole_image_full_cache"] = {"us_per_launch": round(imgf["decode_us_per_launch"], 3),
                                                    "GBs": round(imgf["achieved_GBs"], 1),
                                                    "bytes_per_launch": round(imgf["kv_bytes_per_launch"]),
                                                    "launches": imgf["decode_launches"]}
        print(json.dumps(res), flush=True)
        return 0
    comp = r.run(w, start, steps, args.warmup, *tune, *variant)
    log("compressed, window:", json.dumps(comp))
    full = None if args.skip_full else r.run(w.full_cache(), start, steps, args.warmup, *tune)
    if full:
        log("full cache, window:", json.dumps(full))
        # the two legs of a printed line never do the same work
        assert comp["evicting_lines"] >= 1 and comp["kv_bytes_total"] < full["kv_bytes_total"], "degenerate window"
    comp_img = full_img = None
    if not args.no_whole_image:
        if (start, steps) == (0, N):
            comp_img, full_img = comp, full
        else:
            comp_img = r.run(w, 0, N, args.warmup, *tune, *variant)
            log("compressed, whole image:", json.dumps(comp_img))
            if not args.skip_full:
                full_img = r.run(w.full_cache(), 0, N, args.warmup, *tune)
                log("full cache, whole image:", json.dumps(full_img))

    out = {
        "metric": "decode attn+evict us/step (all layers, compressed cache); HBM GB/s vs peak; speedup vs full cache",
        "value": round(comp["us_per_step"], 2),
        "unit": "us/step",
        "n_gpus": 1,
        "steps": steps,
        "warmup": args.warmup,
        "ms_per_step": round(comp["us_per_step"] / 1e3, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "n_layers": w.n_layers, "sequences": w.batch, "n_heads": w.n_heads,
                   "head_dim": w.head_dim, "n_cond": w.n_cond, "grid": f"{w.n_lines}x{w.line_len}",
                   "budget": w.budget, "n_init": w.n_init, "n_recent_lines": w.n_recent_lines,
                   "score_mode": args.score_mode, "guide_queue": args.guide_queue, "fused_rope": args.fused_rope,
                   "launches": "one decode kernel per layer per token (decode_step_layers), one eviction kernel "
                               "per line for all layers (end_of_line_evict_layers), enqueued back to back on one "
                               "stream, no graph"},
        "window": {"first_step": start, "steps": steps, "steps_requested": requested,
                   "evicting_ends_of_line": comp["evicting_lines"],
                   "mean_keys_compressed": round(comp["mean_keys"], 2),
                   "mean_keys_full": round(full["mean_keys"], 2) if full else None,
                   "reached_by": f"steps 0..{start - 1} of the image run untimed first" if start else
                                 "starts at the first token of the image"},
        "evict_us_per_layer": comp["evict_us_per_layer"],
        "evict_share": round(comp["evict_ms"] / comp["total_ms"], 4),
        "host_wall_ms": round(comp["host_wall_ms"], 1),
        "roofline": {
            "kernel": "decode_attn_kernel (compressed cache), the window's launches",
            "bound": "hbm",
            "achieved": round(comp["achieved_GBs"], 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(comp["achieved_GBs"] / HBM_PEAK_GBS, 4),
            "traffic": None,
            "algorithmic_bytes_per_launch": round(comp["kv_bytes_per_launch"]),
            "us_per_launch": round(comp["decode_us_per_launch"], 3),
            "launches": comp["decode_launches"],
        },
        "cpu_baseline": cpu,
        "cache_memory": cache_memory(w, args.score_mode, args.guide_queue),
        "paper_end_to_end_speedup_context": {"value": PAPER_CONTEXT.get(w.name), "hardware": "NVIDIA A800",
                                             "note": "whole-model generation, not this path"},
    }
    if full:
        out["full_cache"] = {
            "us_per_step": round(full["us_per_step"], 2),
            "achieved_GBs": round(full["achieved_GBs"], 1),
            "frac": round(full["achieved_GBs"] / HBM_PEAK_GBS, 4),
            "us_per_launch": round(full["decode_us_per_launch"], 3),
        }
        out["speedup_vs_full_cache"] = round(full["us_per_step"] / comp["us_per_step"], 3)
        out["byte_ratio_full_over_compressed"] = round(full["kv_bytes_total"] / comp["kv_bytes_total"], 3)
    if comp_img:
        img = whole_image_summary(w, comp_img, full_img)
        out["whole_image"] = img
        out["whole_image_ms"] = img["whole_image_ms"]
        out["us_per_step_first_half"] = img["us_per_step_first_half"]
        out["us_per_step_last_half"] = img["us_per_step_last_half"]
        table = {w.name: img}
        plain = not (args.sequences or args.layers or args.budget_lines or args.score_mode or args.guide_queue or args.fused_rope
                     or args.groups_per_wave or args.n_split)
        if not args.no_table and not args.skip_full and plain:
            del r
            for name in TABLE_WORKLOADS:
                if name in table:
                    continue
                torch.cuda.empty_cache()
                wt = synth.WORKLOADS[name]
                rt = Runner(wt, device)
                c = rt.run(wt, 0, wt.n_visual, args.warmup)
                f = rt.run(wt.full_cache(), 0, wt.n_visual, args.warmup)
                table[name] = whole_image_summary(wt, c, f)
                log(f"{name}:", json.dumps(table[name]))
                del rt
        out["per_workload"] = {k: table[k] for k in TABLE_WORKLOADS if k in table} or table
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
