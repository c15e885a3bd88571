"""decode_step_static (the entry point that allocates nothing: split partials in a device array
inside the library) against decode_step (partials in the caller's workspace), through the C
ABI: two calls in a row on one GPU, the second on a smaller input, so the second call finds the
first one's partials in the array."""
import sys

import pytest
import torch

from paper_2512_04857_amd import binding, synth

pytestmark = pytest.mark.gpu

OUT_TOL = 1e-2      # stated bar for attention outputs (bf16 inputs, fp32 accumulation)
TIGHT_TOL = 2e-4    # what fp32 outputs from identical inputs actually meet


def _reference_and_static(w, n_split, steps, dev):
    """Runs `steps` decode steps of the full-cache workload `w` (prefix of w.n_cond keys) through
    a handle (decode_step) and through decode_step_static on its own copy of the cache."""
    cfg = binding.cfg_from_workload(w)
    ref = binding.LineARCache(cfg, dev)
    kc, vc = synth.cond_kv(w, dev)
    ref.start_image(kc, vc)
    if n_split:
        binding.linear_set_tuning(ref.handle, 0, n_split)
    P, d, C = w.batch * w.n_heads, w.head_dim, w.n_cond
    pitch = C + steps + 3                       # any pitch that holds the rows
    k_own = torch.full((P, pitch, d), float("nan"), dtype=w.torch_dtype, device=dev)
    v_own = torch.full((P, pitch, d), float("nan"), dtype=w.torch_dtype, device=dev)
    k_own[:, :C] = kc[0].reshape(P, C, d)
    v_own[:, :C] = vc[0].reshape(P, C, d)
    out_ref = torch.empty((w.batch, w.n_heads, d), dtype=torch.float32, device=dev)
    out_own = torch.full((P, d), float("nan"), dtype=torch.float32, device=dev)
    dt = binding.LINEAR_BF16 if w.dtype == "bf16" else binding.LINEAR_F32
    worst = 0.0
    stream = ref.stream()
    for step in range(steps):
        q, k, v = synth.step_qkv(w, step, dev)
        ref.decode_step(0, q[0], k[0], v[0], out_ref)
        binding.decode_step_static(dt, d, P, C + step, pitch, k_own.data_ptr(), v_own.data_ptr(),
                                   q[0].data_ptr(), k[0].data_ptr(), v[0].data_ptr(), out_own.data_ptr(),
                                   0.0, n_split, stream)
        torch.cuda.synchronize()
        err = (out_own - out_ref.reshape(P, d)).abs().max().item()
        worst = max(worst, err)
        assert err <= OUT_TOL and err <= TIGHT_TOL, f"{w.name}: step {step}: outputs differ by {err:.3e}"
        # against plain fp32 attention over the rows the step saw
        K = k_own[:, :C + step + 1].float()
        V = v_own[:, :C + step + 1].float()
        logits = torch.einsum("pd,ptd->pt", q[0].reshape(P, d).float(), K) / d ** 0.5
        plain = torch.einsum("pt,ptd->pd", torch.softmax(logits, dim=-1), V)
        assert (out_own - plain).abs().max().item() <= TIGHT_TOL
    kg, vg, _ = ref.gather(0)
    n = C + steps
    assert torch.equal(kg.reshape(P, n, d), k_own[:, :n]) and torch.equal(vg.reshape(P, n, d), v_own[:, :n])
    assert bool(torch.isnan(k_own[:, n:].float()).all())          # rows behind the cache untouched
    ref.close()
    return worst


def test_static_scratch_variant_matches_decode_step_twice_in_a_row():
    dev = "cuda:0"
    assert binding.linear_static_scratch_bytes() == 4 << 20
    # first call: 24 pairs, 600 cached keys of 128 bf16 -> the planner splits them over 9
    # workgroups per pair (few pairs), partials in the library's array
    big = synth.Workload("static-big", 1, 2, 12, 128, 600, 8, 1, 8, 4, 1, "bf16", 41)
    shape = binding.linear_plan_shape(binding.cfg_from_workload(big), 600)
    assert shape["n_split"] > 1
    e1 = _reference_and_static(big, 0, 5, dev)
    # second call, smaller input (6 pairs, 200 keys of 64 fp32), three workgroups per pair forced
    small = synth.Workload("static-small", 1, 1, 6, 64, 200, 8, 1, 8, 4, 1, "f32", 42)
    e2 = _reference_and_static(small, 3, 5, dev)
    # and a third that needs no split at all (one workgroup per pair; the array is not used)
    e3 = _reference_and_static(synth.Workload("static-one", 1, 1, 3, 64, 40, 8, 1, 8, 4, 1, "bf16", 43), 1, 3, dev)
    print(f"decode_step_static vs decode_step: max |diff| {e1:.2e} / {e2:.2e} / {e3:.2e}", file=sys.stderr)


def test_static_variant_empty_cache_and_capacity():
    dev = "cuda:0"
    P, d = 4, 64
    k_own = torch.full((P, 4, d), float("nan"), dtype=torch.bfloat16, device=dev)
    v_own = torch.full((P, 4, d), float("nan"), dtype=torch.bfloat16, device=dev)
    g = torch.Generator(device=dev).manual_seed(20251204)
    q = torch.randn((P, d), device=dev, generator=g).to(torch.bfloat16)
    k = torch.randn((P, d), device=dev, generator=g).to(torch.bfloat16)
    v = torch.randn((P, d), device=dev, generator=g).to(torch.bfloat16)
    out = torch.empty((P, d), dtype=torch.float32, device=dev)
    binding.decode_step_static(binding.LINEAR_BF16, d, P, 0, 4, k_own.data_ptr(), v_own.data_ptr(), q.data_ptr(),
                               k.data_ptr(), v.data_ptr(), out.data_ptr())
    torch.cuda.synchronize()
    # one key: the output is its value row (up to the rounding of exp2 and the division by the sum)
    assert (out - v.float()).abs().max().item() <= 1e-5
    assert torch.equal(k_own[:, 0], k) and torch.equal(v_own[:, 0], v)
    with pytest.raises(binding.LinearError) as e:  # 1024 pairs x 64 splits x 130 floats = 34 MB
        binding.decode_step_static(binding.LINEAR_BF16, 128, 1024, 30000, 30001, 256, 256, 256, 256, 256, 256,
                                   0.0, 64)
    assert e.value.code == binding.LINEAR_ECAPACITY
