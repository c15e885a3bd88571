#!/usr/bin/env python3
"""Benchmark of the LineAR decode path on one MI355X.

A *step* is one decode step of the whole workload: decode_step for every layer (append +
attention + saliency accumulation), plus, when the step closes a raster line,
end_of_line_evict for every layer (selection + compaction).  The timed region starts at
the first token of an image with all inputs resident in HBM and covers K steps (default:
one whole image), for the compressed cache (the headline value) and for the same kernels
on the full cache (B = N).  One JSON line goes to stdout; progress goes to stderr.
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

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published peak
PAPER_CONTEXT = {          # end-to-end speedups the paper prints (Table 4 / Table 1), NVIDIA A800
    "llamagen-xl": 7.57, "janus-pro-7b": 5.62, "janus-pro-1b": 5.87, "lumina-mgpt-768": 2.13}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(w, budget_s: float):
    """The CPU oracle as it stands, one thread, on whole-image replays of slices of a
    one-layer, one-sequence copy of the workload (slices are independent, so the whole
    workload costs slices x this).  Runs before the GPU is touched."""
    import importlib.util

    import torch
    from threadpoolctl import threadpool_limits

    from paper_2512_04857_amd import synth

    spec = importlib.util.spec_from_file_location("linear_oracle", os.path.join(ROOT, "oracle", "linear_oracle.py"))
    o = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(o)
    n_heads = min(w.n_heads, 8)
    ws = synth.shrink(w, n_layers=1, batch=1, n_heads=n_heads)
    torch.set_num_threads(1)
    kc, vc = synth.cond_kv(ws)
    q, k, v = synth.image_qkv(ws)
    f = lambda t: t.to(torch.float64).numpy()
    kc, vc, q, k, v = f(kc[0, 0]), f(vc[0, 0]), f(q[:, 0, 0]), f(k[:, 0, 0]), f(v[:, 0, 0])
    done, t0 = 0, time.perf_counter()
    with threadpool_limits(limits=1):
        while time.perf_counter() - t0 < budget_s:      # whole images only; heads taken in turn
            h = done % n_heads
            o.run_slice(kc[h], vc[h], q[:, h], k[:, h], v[:, h], line_len=w.line_len, n_lines=w.n_lines,
                        budget=w.budget, n_init=w.n_init, n_recent_lines=w.n_recent_lines)
            done += 1
    dt = time.perf_counter() - t0
    total_slices = w.n_layers * w.batch * w.n_heads
    us_per_step = dt / (done * w.n_visual) * total_slices * 1e6
    return {"value": round(us_per_step, 1), "unit": "us/step", "cores": 1, "kind": "oracle",
            "sample": f"{done} whole-image replays ({w.n_visual} steps each) of single (layer, sequence, head) "
                      f"slices in {dt:.1f} s, scaled linearly to the workload's {total_slices} slices"}


def sum_keys(w, steps):
    """Keys read per pair over decode steps [0, steps): closed form of the cache-length
    trajectory (grows to B, then saw-tooths between B-n+1 and B)."""
    C, n, B = w.n_cond, w.line_len, w.budget
    tot = 0
    for i in range(1, steps + 1):
        vis = i if i <= B else B - n + ((i - 1) % n) + 1
        tot += C + vis
    return tot


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

    def run(self, wl, steps, warmup, groups_per_wave=0, n_split=0, score_mode=0, guide_queue=0, fused_rope=False):
        """Times `steps` decode steps of workload variant `wl` (same shapes, its own budget)
        from the start of an image.  Returns a dict of measurements."""
        torch, binding = self.torch, self.binding
        L, n = wl.n_layers, wl.line_len
        cache = binding.LineARCache(binding.cfg_from_workload(wl, score_mode=score_mode, guide_queue=guide_queue),
                                    self.device)
        lib = binding.lib()
        dsteps, evicts = lib.decode_step_layers, lib.end_of_line_evict_layers
        if fused_rope:
            # the rotary embedding fused into the step: the pre-generated q, k stand in for unrotated
            # ones (the timing does not depend on the values); one table row per position
            from paper_2512_04857_amd import synth
            table = torch.stack([synth.rope_cos_sin(wl, wl.n_cond + i, self.device) for i in range(wl.n_visual)])
            tb, tst = table.data_ptr(), table[0].numel() * 4
            rope = lib.decode_step_rope_layers
        qb, kb, vb, ob = self.q.data_ptr(), self.k.data_ptr(), self.v.data_ptr(), self.out.data_ptr()
        st, ost = self.stride, self.ostride
        stream = cache.stream()

        def image(n_steps, events):
            cache.start_image(self.kc, self.vc)
            h = cache.handle
            if groups_per_wave or n_split:
                binding.linear_set_tuning(h, groups_per_wave, n_split)
            if events is not None:
                torch.cuda.synchronize()
                events.append(("start", torch.cuda.Event(enable_timing=True)))
                events[-1][1].record()
            for s in range(n_steps):
                off = s * L * st
                if fused_rope:
                    rc = rope(h, 0, L, qb + off, kb + off, vb + off, tb + s * tst, ob, st, ost, stream)
                else:
                    rc = dsteps(h, 0, L, qb + off, kb + off, vb + off, ob, st, ost, stream)
                if rc:
                    raise binding.LinearError(rc, "decode_step_layers")
                if (s + 1) % n == 0:
                    if events is not None:
                        e = torch.cuda.Event(enable_timing=True)
                        e.record()
                        events.append(("decode_end", e))
                    rc = evicts(h, 0, L, stream)
                    if rc:
                        raise binding.LinearError(rc, "end_of_line_evict_layers")
                    if events is not None:
                        e = torch.cuda.Event(enable_timing=True)
                        e.record()
                        events.append(("line_end", e))
            if events is not None:
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                events.append(("stop", e))
                self.enqueue_s = time.perf_counter()
                torch.cuda.synchronize()

        image(min(warmup, wl.n_visual), None)
        torch.cuda.synchronize()
        ev = []
        t0 = time.perf_counter()
        image(steps, ev)
        wall = time.perf_counter() - t0
        enqueue = self.enqueue_s - t0
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
                if dt > 0 and steps % n:
                    line_ms.append(dt)
            prev = e
        full_lines = steps // n
        half = full_lines // 2
        first = sum(line_ms[:half]) / (half * n) * 1e3 if half else None
        last = sum(line_ms[full_lines - half:full_lines]) / (half * n) * 1e3 if half else None
        compresses = wl.budget < wl.n_visual
        evict_lines = [ln for ln in range(1, full_lines + 1)
                       if compresses and wl.budget // n <= ln <= wl.n_lines - 1]
        keys = sum_keys(wl, steps)
        tok_bytes = 2 * wl.n_heads * wl.head_dim * self.q.element_size() * wl.batch
        launches = steps * L
        return {
            "us_per_step": total_ms * 1e3 / steps,
            "total_ms": total_ms,
            "host_wall_ms": wall * 1e3,
            "host_enqueue_ms": enqueue * 1e3,
            "decode_ms": decode_ms,
            "evict_ms": evict_ms,
            "us_per_step_first_half": first,
            "us_per_step_last_half": last,
            "decode_launches": launches,
            "decode_us_per_launch": decode_ms * 1e3 / launches,
            "evict_layer_lines": len(evict_lines) * L,      # evictions of one layer; layers share launches
            "evict_us_per_layer": (evict_ms * 1e3 / (len(evict_lines) * L)) if evict_lines else None,
            "kv_bytes_per_launch": keys * tok_bytes / steps,
            "kv_bytes_total": keys * tok_bytes * L,
            "mean_keys": keys / steps,
            "line_us_per_launch": [round(x * 1e3 / (n * L), 2) for x in line_ms],
        }


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


def read_traffic(name):
    """HBM bytes per decode launch measured with rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE,
    scaled by a copy kernel of known size), if a summary for this workload is committed."""
    path = os.path.join(ROOT, "profiles", f"decode_attn_{name}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="decode steps to time (default: one whole image)")
    ap.add_argument("--warmup", type=int, default=48)
    ap.add_argument("--workload", default="llamagen-xl")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="0 skips the CPU oracle leg")
    ap.add_argument("--skip-full", action="store_true", help="do not time the full-cache variant")
    ap.add_argument("--calibrate-copy-mib", type=int, default=0,
                    help="also run one elementwise read+write pass over this many MiB (a traffic yardstick for "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs)")
    ap.add_argument("--sequences", type=int, default=0,
                    help="override the number of sequences (e.g. 512 = the paper's Table 4 batch of 256 "
                         "with both guidance halves, for the LlamaGen-XL shape)")
    ap.add_argument("--budget-lines", type=int, default=0,
                    help="override the budget B, in raster lines (rho sweeps: 6 of 24 lines = 1/4, ...)")
    ap.add_argument("--score-mode", type=int, default=0,
                    help="0 = Eq. 9 as printed (default), 1 = decode-softmax mass, 2 = accumulated attention")
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

    from paper_2512_04857_amd import synth

    w = synth.WORKLOADS[args.workload]
    from dataclasses import replace
    if args.sequences:
        w = replace(w, batch=args.sequences, name=f"{w.name}-seq{args.sequences}")
    if args.budget_lines:
        w = replace(w, budget=args.budget_lines * w.line_len, name=f"{w.name}-b{args.budget_lines}")
    steps = args.steps or w.n_visual
    if steps > w.n_visual:
        print(f"bench.py: --steps is capped at one image ({w.n_visual} decode steps)", file=sys.stderr)
        steps = w.n_visual

    cpu = cpu_baseline(w, args.cpu_seconds) if args.cpu_seconds > 0 else None
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
    comp = r.run(w, steps, args.warmup, args.groups_per_wave, args.n_split, args.score_mode, args.guide_queue,
                 args.fused_rope)
    log("compressed:", json.dumps(comp))
    full = None if args.skip_full else r.run(w.full_cache(), steps, args.warmup, args.groups_per_wave, args.n_split)
    if full:
        log("full cache:", json.dumps(full))

    achieved = comp["kv_bytes_per_launch"] / (comp["decode_us_per_launch"] * 1e-6) / 1e9
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
        "whole_image_ms": round(comp["total_ms"], 3) if steps == w.n_visual else None,
        "us_per_step_first_half": comp["us_per_step_first_half"],
        "us_per_step_last_half": comp["us_per_step_last_half"],
        "evict_us_per_layer": comp["evict_us_per_layer"],
        "evict_share": round(comp["evict_ms"] / comp["total_ms"], 4),
        "host_wall_ms": round(comp["host_wall_ms"], 1),
        "roofline": {
            "kernel": "decode_attn_kernel (compressed cache)",
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": read_traffic(w.name),
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
        fa = full["kv_bytes_per_launch"] / (full["decode_us_per_launch"] * 1e-6) / 1e9
        out["full_cache"] = {
            "us_per_step": round(full["us_per_step"], 2),
            "whole_image_ms": round(full["total_ms"], 3) if steps == w.n_visual else None,
            "us_per_step_first_half": full["us_per_step_first_half"],
            "us_per_step_last_half": full["us_per_step_last_half"],
            "achieved_GBs": round(fa, 1),
            "frac": round(fa / HBM_PEAK_GBS, 4),
            "us_per_launch": round(full["decode_us_per_launch"], 3),
        }
        out["speedup_vs_full_cache"] = round(full["us_per_step"] / comp["us_per_step"], 3)
        out["byte_ratio_full_over_compressed"] = round(full["kv_bytes_total"] / comp["kv_bytes_total"], 3)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
