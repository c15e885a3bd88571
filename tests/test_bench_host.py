"""Host-side parts of bench.py that need no GPU: the algorithmic-byte accounting against closed
forms, the placement of the timed window, the cache-memory accounting, the one-GPU rule and the
CPU-oracle leg."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from paper_2512_04857_amd import synth  # noqa: E402

BENCH_WORKLOADS = ["tiny-a", "tiny-b", "tiny-c", "llamagen-xl", "janus-pro-1b", "janus-pro-7b", "lumina-mgpt-768",
                   "lumina-mgpt-1024"]


def closed_form_keys(w):
    """Sum over the image of the keys one query reads: all N steps see the C conditional keys;
    the visual part grows 1..B during the first B steps and then repeats B-n+1..B on every one
    of the remaining h - B/n lines (Sec. 3.3: B - n retained after each eviction plus the line
    being written)."""
    C, n, h, B = w.n_cond, w.line_len, w.n_lines, w.budget
    N = n * h
    grow = B * (B + 1) // 2
    saw = (h - B // n) * (n * (B - n) + n * (n + 1) // 2)
    return N * C + grow + saw


@pytest.mark.parametrize("name", ["tiny-a", "llamagen-xl", "janus-pro-1b", "janus-pro-7b", "lumina-mgpt-768"])
def test_keys_read_per_image_match_the_closed_form(name):
    w = synth.WORKLOADS[name]
    assert bench.sum_keys(w, w.n_visual) == closed_form_keys(w)
    wf = w.full_cache()
    N, C = w.n_visual, w.n_cond
    assert bench.sum_keys(wf, N) == N * C + N * (N + 1) // 2       # causal attention over everything
    # a window is a slice of the same trajectory
    assert bench.sum_keys(w, 10, 0) + bench.sum_keys(w, N - 10, 10) == closed_form_keys(w)


def test_byte_ratios_of_the_benchmark_workloads():
    """Full-cache over compressed K/V bytes per image: 3.64 / 2.47 / 2.02 / 2.81."""
    want = {"llamagen-xl": 3.642, "janus-pro-1b": 2.474, "janus-pro-7b": 2.017, "lumina-mgpt-768": 2.805}
    for name, r in want.items():
        w = synth.WORKLOADS[name]
        got = bench.sum_keys(w.full_cache(), w.n_visual) / bench.sum_keys(w, w.n_visual)
        assert abs(got - r) < 1e-3, (name, got)


@pytest.mark.parametrize("name", BENCH_WORKLOADS)
def test_timed_window_is_never_degenerate(name):
    """Whatever --steps asks for, the timed window holds the end-of-line call of an evicting
    line, its compressed leg reads fewer keys than its full-cache leg, and -- when the image is
    long enough -- it starts behind the first eviction, where the cache has reached its
    steady-state length."""
    w = synth.WORKLOADS[name]
    n, N, h, B = w.line_len, w.n_visual, w.n_lines, w.budget
    for asked in sorted({1, 2, 5, 20, n - 1, n, n + 1, 3 * n, N - n, N - 1, N, N + 7}):
        start, steps = bench.steady_window(w, asked)
        assert 0 <= start and start + steps <= N and steps >= min(max(asked, 1), N)
        ends = bench.evicting_ends_in(w, start, steps)
        assert ends, (name, asked, start, steps)
        assert all(B // n <= l <= h - 1 for l in ends)
        comp, full = bench.sum_keys(w, steps, start), bench.sum_keys(w.full_cache(), steps, start)
        assert comp < full, (name, asked)
        if asked >= N:
            assert (start, steps) == (0, N)
        elif start > 0:      # (a window longer than the evicting part of the image starts at token 0)
            assert (start + steps) % n == 0 and bench.evicting_line(w, (start + steps) // n)   # ends with an eviction
        if steps <= (h - 1 - B // n) * n:
            assert start >= (B // n) * n          # behind the first eviction: every step sees > B - n visual keys
            assert all(bench.visual_len_at(w, s) > B - n for s in range(start, start + steps))
    # the driver's invocation on the headline workload
    if name == "llamagen-xl":
        assert bench.steady_window(w, 20) == (100, 20)


def test_window_of_a_workload_that_never_evicts_is_the_image_prefix():
    wf = synth.LLAMAGEN_XL.full_cache()
    assert bench.steady_window(wf, 20) == (0, 20) and bench.evicting_ends_in(wf, 0, wf.n_visual) == []


def test_cache_memory_accounting():
    w = synth.LLAMAGEN_XL
    m = bench.cache_memory(w, 0)
    per_token = 2 * w.n_layers * w.batch * w.n_heads * w.head_dim * 2      # K and V, bf16, every layer
    assert m["compressed_kv_bytes"] == per_token * (w.n_cond + w.budget)
    assert m["full_kv_bytes"] == per_token * (w.n_cond + w.n_visual)
    assert 0 < m["compressed_scratch_bytes"] < m["compressed_kv_bytes"]
    assert 0.75 < m["saving"] < 1 - (w.n_cond + w.budget) / (w.n_cond + w.n_visual) + 1e-9


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0 and "one GPU" in p.stderr and p.stdout.strip() == ""


def test_a_budget_that_holds_the_whole_image_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--budget-lines", "24", "--cpu-seconds", "0"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0 and "same work" in p.stderr and p.stdout.strip() == ""


def test_cpu_oracle_leg_uses_the_cores_and_says_how_many():
    w = synth.TINY_B
    r = bench.cpu_baseline(w, w.name, {}, 1.0)
    assert r["kind"] == "oracle" and r["unit"] == "us/step"
    assert 1 <= r["cores"] <= 16 and r["cores"] <= r["cores_visible"]
    assert r["value"] > 0 and abs(r["single_core_us_per_step"] / r["cores"] - r["value"]) <= 0.11
    assert "replays" in r["sample"]
