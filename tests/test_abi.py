"""Host-side checks that need no GPU: the library loads, exports every entry point the
header declares, and rejects invalid configurations and arguments with error codes."""
import ctypes
import os
import re

import pytest

from paper_2512_04857_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_entry_points():
    names = []
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            names += re.findall(r"LINEAR_API\s+[\w\s\*]+?\b(\w+)\s*\(", text)
    return names


def test_library_exports_every_declared_symbol():
    names = declared_entry_points()
    assert set(names) == set(binding.EXPORTS) and len(names) == len(binding.EXPORTS)
    L = binding.lib()
    for n in names:
        assert getattr(L, n) is not None


def good(**over):
    w = synth.LLAMAGEN_XL
    kw = dict(n_layers=2, batch=2, n_heads=4, head_dim=w.head_dim, n_cond=w.n_cond,
              line_len=w.line_len, n_lines=w.n_lines, budget=w.budget, n_init=w.n_init,
              n_recent_lines=w.n_recent_lines, dtype="bf16")
    kw.update(over)
    return binding.make_cfg(**kw)


def test_workspace_sizes():
    cfg = good()
    cache, scratch = binding.linear_workspace_bytes(cfg)
    assert cache == 2 * 4 * (1 + 96) * 64 * 2
    # accumulators + position maps + partials + mid logits + counters, 256-byte aligned parts
    assert scratch >= 2 * 8 * 48 * 4 + 2 * 8 * 97 * 4 and scratch % 256 == 0
    full = good(budget=576)
    cache_full, _ = binding.linear_workspace_bytes(full)
    assert cache_full == 2 * 4 * 577 * 64 * 2
    for w in synth.WORKLOADS.values():
        binding.linear_workspace_bytes(binding.cfg_from_workload(w))


@pytest.mark.parametrize("over", [
    dict(head_dim=96), dict(head_dim=0), dict(budget=100), dict(budget=0), dict(budget=600),
    dict(n_init=49), dict(n_recent_lines=0), dict(n_recent_lines=3), dict(dtype=7),
    dict(n_layers=0), dict(batch=0), dict(n_cond=-1), dict(line_len=0), dict(score_mode=4), dict(score_mode=-1), dict(score_mode=3, guide_queue=1), dict(out_dtype=2), dict(out_dtype=-1), dict(guide_queue=3), dict(guide_queue=-1),
    dict(guide_queue=2, score_mode=1), dict(guide_queue=2, score_mode=2),
    dict(scale=-1.0), dict(scale=float("nan")), dict(scale=float("inf")),
    dict(line_len=1, n_lines=100000, budget=50000, n_init=0),     # mid larger than the ranking limit
    dict(score_mode=2, line_len=16, n_lines=1024, budget=7712, n_init=16, n_recent_lines=400),  # > 7680 scored slots
])
def test_invalid_configurations_are_rejected(over):
    with pytest.raises(binding.LinearError) as e:
        binding.linear_workspace_bytes(good(**over))
    assert e.value.code == binding.LINEAR_EINVAL


def test_largest_accumulated_attention_configuration_fits_the_decode_step():
    """Score mode 2 stages B - N_init logits per step in LDS beside the softmax partials of up to
    16 wavefronts: the largest accepted configuration keeps that within 64 KiB."""
    cfg = good(score_mode=2, line_len=16, n_lines=1024, budget=7696, n_init=16, n_recent_lines=400)
    binding.linear_workspace_bytes(cfg)                     # 7680 scored slots: accepted
    workers_bytes = (16 * 8 * (64 + 1) + 16) * 4            # d = 64 bf16: 8 softmax workers per wavefront
    assert workers_bytes + 7680 * 4 <= 64 * 1024
    assert (16 * 4 * (128 + 1) + 16) * 4 + 7680 * 4 <= 64 * 1024   # d = 128


def test_null_and_alignment_errors_without_touching_the_gpu():
    L = binding.lib()
    cfg = good()
    h = ctypes.c_void_p()
    assert L.kv_init(None, None, None, None, None, None, None, ctypes.byref(h)) == binding.LINEAR_ENULL
    two = (ctypes.c_void_p * 2)(256, 512)
    odd = (ctypes.c_void_p * 2)(256, 520)
    assert L.kv_init(ctypes.byref(cfg), two, two, 4096, None, None, None, ctypes.byref(h)) == binding.LINEAR_ENULL
    assert L.kv_init(ctypes.byref(cfg), two, odd, 4096, two, two, None, ctypes.byref(h)) == binding.LINEAR_EALIGN
    assert L.kv_init(ctypes.byref(cfg), two, two, 4100, two, two, None, ctypes.byref(h)) == binding.LINEAR_EALIGN
    assert L.decode_step(None, 0, 16, 16, 16, 16, None) == binding.LINEAR_ENULL
    assert L.decode_step_rope(None, 0, 16, 16, 16, 16, 16, None) == binding.LINEAR_ENULL
    assert L.decode_step_rope(8, 0, 16, 16, 16, None, 16, None) == binding.LINEAR_ENULL      # no table
    assert L.decode_step_rope(8, 0, 16, 16, 16, 20, 16, None) == binding.LINEAR_EALIGN       # table not 16-byte aligned
    assert L.decode_step_rope_layers(8, 0, 1, 16, 16, 16, None, 16, 128, 256, None) == binding.LINEAR_ENULL
    assert L.end_of_line_evict(None, 0, None) == binding.LINEAR_ENULL
    assert L.kv_gather(None, 0, None, None, None, None, None) == binding.LINEAR_ENULL
    assert L.kv_free(None) == binding.LINEAR_OK
    assert L.linear_strerror(binding.LINEAR_ESTATE).decode().startswith("call not allowed")
    assert L.linear_strerror(-99).decode() == "unknown error"


def test_static_step_argument_errors_without_touching_the_gpu():
    """decode_step_static checks its arguments and the capacity of the library's own scratch
    array before any device call."""
    L = binding.lib()
    ok = dict(dtype=1, d=128, P=8, T=100, pitch=128)

    def call(dtype=1, d=128, P=8, T=100, pitch=128, kc=256, vc=256, q=256, k=256, v=256, scale=0.0, ns=0, out=256):
        return L.decode_step_static(dtype, d, P, T, pitch, kc, vc, q, k, v, scale, ns, out, None)

    assert call(kc=None) == binding.LINEAR_ENULL and call(out=None) == binding.LINEAR_ENULL
    assert call(q=264) == binding.LINEAR_EALIGN
    for bad in (dict(dtype=2), dict(d=96), dict(P=0), dict(T=-1), dict(pitch=100), dict(scale=-1.0),
                dict(scale=float("inf")), dict(ns=65), dict(ns=-1), dict(T=2_000_000, pitch=2_000_001)):
        assert call(**bad) == binding.LINEAR_EINVAL, bad
    # 1024 pairs x 64 workgroups x (128 + 2) floats = 34 MB of partials: more than the array holds
    assert call(P=1024, T=30000, pitch=30001, ns=64) == binding.LINEAR_ECAPACITY
    assert "static scratch" in L.linear_strerror(binding.LINEAR_ECAPACITY).decode()
    assert L.linear_static_scratch_bytes(None) == binding.LINEAR_ENULL


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "liblinear_kv.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.lib()


DEPTHS = {1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 14, 16}


@pytest.mark.parametrize("name", sorted(synth.WORKLOADS))
@pytest.mark.parametrize("full,guide_queue", [(False, binding.LINEAR_QUEUE_AUTO), (True, binding.LINEAR_QUEUE_AUTO),
                                             (False, binding.LINEAR_QUEUE_LOGITS)],
                         ids=["compressed", "full-cache", "compressed-logits-queue"])
def test_launch_shape_covers_every_step(name, full, guide_queue):
    """Host planner: for every cache length a workload reaches (compressed and full cache),
    the decode kernel's launch shape holds all cached keys, leaves no workgroup empty, uses an
    instantiated depth within the register budget, and names a valid wavefront for the new
    token."""
    w = synth.WORKLOADS[name]
    w = w.full_cache() if full else w
    cfg = binding.cfg_from_workload(w, guide_queue=guide_queue)
    t_max = w.n_cond + w.budget
    for gpw, ns in ((0, 0), (1, 0), (5, 0), (16, 0), (0, 3), (3, 7)):
        for keys in range(0, t_max):
            p = binding.linear_plan_shape(cfg, keys, gpw, ns)
            rpg = p["keys_per_group"]
            assert p["keys_per_workgroup"] % rpg == 0
            assert p["n_split"] * p["keys_per_workgroup"] >= keys
            assert p["n_split"] == 1 or (p["n_split"] - 1) * p["keys_per_workgroup"] < keys
            assert p["depth"] in DEPTHS
            assert 1 <= p["n_waves"] <= (16 if p["depth"] <= 8 else 12)
            assert p["n_waves"] * p["depth"] * rpg >= p["keys_per_workgroup"]
            assert 0 <= p["new_wave"] < p["n_waves"]
            if ns:
                assert p["n_split"] <= max(ns, -(-keys // (128 * rpg)))
            last = keys - (p["n_split"] - 1) * p["keys_per_workgroup"]
            assert p["new_wave"] == -(-last // rpg) % p["n_waves"]
    with pytest.raises(binding.LinearError):
        binding.linear_plan_shape(cfg, t_max, 0, 0)
