"""Host-side parts of bench.py that need no GPU: the algorithmic-byte accounting against closed
forms, the cache-memory accounting, the one-GPU rule and the traffic figure's source."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from paper_2512_04857_amd import synth  # noqa: E402


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


def test_byte_ratios_of_the_benchmark_workloads():
    """Full-cache over compressed K/V bytes per image: 3.64 / 2.47 / 2.02 / 2.81."""
    want = {"llamagen-xl": 3.642, "janus-pro-1b": 2.474, "janus-pro-7b": 2.017, "lumina-mgpt-768": 2.805}
    for name, r in want.items():
        w = synth.WORKLOADS[name]
        got = bench.sum_keys(w.full_cache(), w.n_visual) / bench.sum_keys(w, w.n_visual)
        assert abs(got - r) < 1e-3, (name, got)


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


def test_traffic_figure_comes_from_the_committed_profile():
    v = bench.read_traffic("llamagen-xl")
    assert v is None or 1e6 < v < 1e9
    assert bench.read_traffic("no-such-workload") is None
