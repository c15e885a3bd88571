"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the
same seeded inputs (rules in parity_harness.py)."""
import sys

import pytest
import torch

from paper_2512_04857_amd import binding, synth
from parity_harness import all_slices, run_parity, sampled_slices

pytestmark = pytest.mark.gpu

W = synth.Workload
# Small shapes the oracle finishes in seconds that still span several 128-key tiles, split
# boundaries inside the mid region, ragged tails, pair counts that are not multiples of 8.
MID_SPLIT = W("mid-split", 2, 3, 5, 64, 40, 24, 8, 96, 24, 1, "bf16", 21)
LUMINA_SLICE = W("lumina-slice", 1, 2, 3, 128, 256, 49, 9, 294, 49, 1, "bf16", 22)
F32_R2 = W("f32-r2", 1, 2, 2, 128, 5, 10, 7, 40, 7, 2, "f32", 23)
FULL_SPLIT = W("full-split", 1, 2, 3, 64, 3, 24, 12, 288, 24, 1, "bf16", 24)
NO_COND = W("no-cond", 1, 1, 8, 64, 0, 8, 9, 32, 0, 1, "bf16", 25)
F32_D64_LONG = W("f32-d64-long", 1, 1, 2, 64, 130, 16, 6, 64, 16, 1, "f32", 26)
STREAMING = W("bf16-streaming", 1, 2, 2, 128, 7, 12, 6, 36, 12, 1, "bf16", 27)   # mid == n
# 264 rows of 512 B may move at an end of line: more than the register-resident eviction
# kernel holds, so this one runs the tiled kernel.
F32_WIDE = W("f32-wide", 1, 1, 2, 128, 3, 64, 7, 320, 56, 1, "f32", 28)
ONE_TOKEN_LINES = W("one-token-lines", 1, 2, 2, 64, 2, 1, 12, 4, 1, 1, "bf16", 29)   # n = 1: evicts every step
NO_ANCHOR_R3 = W("no-anchor-r3", 2, 1, 3, 64, 0, 6, 9, 36, 0, 3, "f32", 30)          # N_init = 0, r = 3


def say(msg):
    print(msg, file=sys.stderr, flush=True)


@pytest.mark.parametrize("w", [synth.TINY_A, synth.TINY_B, synth.TINY_C], ids=lambda w: w.name)
@pytest.mark.parametrize("score_mode", [0, 1, 2, 3])
def test_tiny_every_slice(w, score_mode):
    rep = run_parity(w, all_slices(w), score_mode=score_mode, random_seed=77)
    say(f"{w.name} mode {score_mode}: {rep}")
    assert rep.steps == 64 and rep.evictions == (w.n_lines - w.budget // w.line_len) * w.n_heads


def test_tiny_full_budget_never_evicts():
    w = synth.TINY_A.full_cache()
    rep = run_parity(w, all_slices(w))
    assert rep.evictions == 0 and rep.steps == 64


# (workload, row groups per wavefront, forced splits, score mode): single-launch shapes with
# 1..16 wavefronts and all three register depths, and split shapes (two launches) whose split
# boundaries fall inside the mid region.
@pytest.mark.parametrize("w,gpw,n_split,score_mode", [
    (MID_SPLIT, 0, 0, 0), (MID_SPLIT, 1, 0, 1), (MID_SPLIT, 16, 0, 0), (MID_SPLIT, 3, 2, 0),
    (MID_SPLIT, 0, 3, 1), (LUMINA_SLICE, 0, 0, 0), (LUMINA_SLICE, 12, 1, 0), (LUMINA_SLICE, 4, 5, 0),
    (LUMINA_SLICE, 0, 2, 1), (F32_R2, 0, 0, 0), (F32_R2, 2, 2, 0), (FULL_SPLIT, 0, 0, 0),
    (FULL_SPLIT, 16, 1, 0), (FULL_SPLIT, 5, 3, 0), (NO_COND, 0, 0, 0), (NO_COND, 1, 0, 0),
    (F32_D64_LONG, 0, 0, 0), (F32_D64_LONG, 8, 2, 1), (STREAMING, 0, 0, 0), (F32_WIDE, 0, 0, 0),
    (ONE_TOKEN_LINES, 0, 0, 0), (ONE_TOKEN_LINES, 0, 0, 1), (NO_ANCHOR_R3, 0, 0, 0), (NO_ANCHOR_R3, 2, 2, 1),
    # accumulated attention (score mode 2): scored range grows with the line, crosses splits
    (MID_SPLIT, 0, 0, 2), (MID_SPLIT, 3, 2, 2), (LUMINA_SLICE, 0, 0, 2), (LUMINA_SLICE, 4, 5, 2),
    (F32_R2, 0, 0, 2), (NO_COND, 1, 0, 2), (ONE_TOKEN_LINES, 0, 0, 2), (NO_ANCHOR_R3, 0, 0, 2),
    (F32_WIDE, 0, 0, 2), (STREAMING, 0, 0, 2),
], ids=lambda x: getattr(x, "name", str(x)))
def test_mid_sizes_every_slice(w, gpw, n_split, score_mode):
    rep = run_parity(w, all_slices(w), groups_per_wave=gpw, n_split=n_split, score_mode=score_mode)
    say(f"{w.name} groups/wave {gpw} splits {n_split} mode {score_mode}: {rep}")
    assert rep.steps == w.n_visual


# Score mode 0 queues the queries by default (Eq. 8 as printed; Eq. 9 is then a matrix product
# at the end of the line, the oracle's own formulation), so the tests above cover that path:
# bf16 and fp32 operands, both head sizes, one and several workgroups per pair, query tiles that
# are full, ragged and single-row, mid regions that are not a multiple of the 16-key tile.
# These run mode 0 with the other queue, the decode step's own logits.
@pytest.mark.parametrize("w,gpw,n_split", [
    (synth.TINY_A, 0, 0), (synth.TINY_B, 0, 0), (synth.TINY_C, 0, 0),
    (MID_SPLIT, 0, 0), (MID_SPLIT, 3, 2), (LUMINA_SLICE, 0, 0), (LUMINA_SLICE, 4, 5), (F32_R2, 0, 0),
    (F32_R2, 2, 2), (NO_COND, 1, 0), (F32_D64_LONG, 0, 0), (STREAMING, 0, 0), (F32_WIDE, 0, 0),
    (ONE_TOKEN_LINES, 0, 0), (NO_ANCHOR_R3, 0, 0),
], ids=lambda x: getattr(x, "name", str(x)))
def test_logits_queue_every_slice(w, gpw, n_split):
    rep = run_parity(w, all_slices(w), groups_per_wave=gpw, n_split=n_split,
                     guide_queue=binding.LINEAR_QUEUE_LOGITS)
    say(f"{w.name} logits queue, groups/wave {gpw} splits {n_split}: {rep}")
    assert rep.steps == w.n_visual


# The rotary embedding fused into the step: q and k go in unrotated, the oracle receives an
# unfused fp32 rotation of the same values from the input generator.  bf16 and fp32, 8 / 16 / 32
# lanes per row, one and several workgroups per pair; the retained K rows must come back with
# exactly the generator's bits.
@pytest.mark.parametrize("w,gpw,n_split,score_mode", [
    (synth.TINY_B, 0, 0, 0), (MID_SPLIT, 0, 0, 0), (MID_SPLIT, 3, 2, 1), (LUMINA_SLICE, 4, 5, 0),
    (F32_R2, 2, 2, 0), (F32_D64_LONG, 0, 0, 2), (NO_COND, 1, 0, 0), (STREAMING, 0, 0, 0),
], ids=lambda x: getattr(x, "name", str(x)))
def test_fused_rope_every_slice(w, gpw, n_split, score_mode):
    rep = run_parity(w, all_slices(w), groups_per_wave=gpw, n_split=n_split, score_mode=score_mode,
                     fused_rope=True)
    say(f"{w.name} fused rope, groups/wave {gpw} splits {n_split} mode {score_mode}: {rep}")
    assert rep.steps == w.n_visual


# `out` in the storage type (what the output projection consumes), laid out [Bz, H d]: single
# launch, split launches (the merge kernel writes it) and the fused-rope step; fp32 storage keeps
# fp32 results.
@pytest.mark.parametrize("w,gpw,n_split,kw", [
    (MID_SPLIT, 0, 0, {}), (MID_SPLIT, 3, 2, {}), (LUMINA_SLICE, 4, 5, dict(fused_rope=True)),
    (FULL_SPLIT, 5, 3, {}), (F32_R2, 2, 2, {}), (NO_COND, 1, 0, dict(score_mode=1)),
], ids=lambda x: getattr(x, "name", str(x)))
def test_output_in_the_storage_type_every_slice(w, gpw, n_split, kw):
    rep = run_parity(w, all_slices(w), groups_per_wave=gpw, n_split=n_split, out_elem=True, **kw)
    say(f"{w.name} out in {w.dtype}, groups/wave {gpw} splits {n_split} {kw}: {rep}")
    assert rep.steps == w.n_visual
    if w.dtype == "bf16":
        assert 1e-5 < rep.max_out_err <= 1e-2          # rounded to bf16, and only that


def test_full_size_output_in_the_storage_type():
    w = synth.JANUS_PRO_1B
    rep = run_parity(w, _sample(w, n_heads=2), layers_call=True, out_elem=True)
    say(f"{w.name} out in bf16: {rep}")
    assert rep.steps == w.n_visual and 1e-5 < rep.max_out_err <= 1e-2


def test_full_size_fused_rope_sampled_slices():
    w = synth.LLAMAGEN_XL
    rep = run_parity(w, _sample(w, n_heads=2), layers_call=True, fused_rope=True)
    say(f"{w.name} fused rope: {rep}")
    assert rep.steps == w.n_visual and rep.evictions == 20 * len(_sample(w, n_heads=2))



def _sample(w, n_heads=None):
    """Sampled (layer, sequence, head) slices of a full-size workload: the first and the last
    layer x the first, a middle and the last sequence x every head (or `n_heads` spread ones)."""
    heads = list(range(w.n_heads))
    if n_heads is not None:
        heads = sorted({0, w.n_heads // 3, w.n_heads // 2, w.n_heads - 1})[:n_heads]
    return sampled_slices(w, sorted({0, w.n_layers - 1}), sorted({0, w.batch // 2, w.batch - 1}), heads)


def _lumina_sample(w):
    """Lumina-shaped images cost the oracle 1.4 s per slice: every head of the last sequence in the
    last layer, and four spread heads for the other (layer, sequence) corners and the middle."""
    corners = [(l, b) for l in (0, w.n_layers - 1) for b in (0, w.batch // 2, w.batch - 1)]
    sl = [(w.n_layers - 1, w.batch - 1, h) for h in range(w.n_heads)]
    sl += [(l, b, h) for (l, b) in corners[:-1] for h in (0, 10, 16, w.n_heads - 1)]
    return sl


@pytest.mark.parametrize("w", [synth.LLAMAGEN_XL, synth.JANUS_PRO_1B, synth.JANUS_PRO_7B,
                               synth.LUMINA_768], ids=lambda w: w.name)
def test_full_size_compressed_sampled_slices(w):
    """The benchmark's shapes and launch configuration; the oracle replays whole images
    for sampled (layer, sequence, head) slices, which is exact because slices never
    interact."""
    sl = _lumina_sample(w) if w is synth.LUMINA_768 else _sample(w)
    rep = run_parity(w, sl, progress=say if w.n_lines > 30 else None, layers_call=True)
    say(f"{w.name}: {len(sl)} slices: {rep}")
    assert rep.steps == w.n_visual
    assert rep.evictions == (w.n_lines - w.budget // w.line_len) * len(sl)


# The budgets of the paper's efficiency table (Table 4) other than the benchmark's: rho = 1/4 for the
# N = 576 models (B = 144: 96 candidates per eviction, 72 survive -- more than one wavefront ranks) and
# rho = 1/6 for N = 2352 (B = 392: 294 candidates); they take other launch plans and end-of-line shapes.
@pytest.mark.parametrize("w,budget,heads", [(synth.LLAMAGEN_XL, 144, None), (synth.JANUS_PRO_7B, 144, 4),
                                            (synth.LUMINA_768, 392, 1)], ids=lambda x: getattr(x, "name", str(x)))
def test_full_size_table4_budgets_sampled_slices(w, budget, heads):
    from dataclasses import replace
    wb = replace(w, budget=budget, name=f"{w.name}-B{budget}")
    sl = _sample(wb, n_heads=heads)
    rep = run_parity(wb, sl, progress=say if w.n_lines > 30 else None, layers_call=True)
    say(f"{wb.name}: {len(sl)} slices: {rep}")
    assert rep.steps == w.n_visual
    assert rep.evictions == (w.n_lines - budget // w.line_len) * len(sl)


@pytest.mark.parametrize("w", [synth.LLAMAGEN_XL, synth.JANUS_PRO_7B, synth.LUMINA_768], ids=lambda w: w.name)
def test_full_size_logits_queue_sampled_slices(w):
    sl = _sample(w, n_heads=2 if w is not synth.LUMINA_768 else 1)
    rep = run_parity(w, sl, guide_queue=binding.LINEAR_QUEUE_LOGITS,
                     progress=say if w.n_lines > 30 else None, layers_call=True)
    say(f"{w.name} logits queue: {len(sl)} slices: {rep}")
    assert rep.steps == w.n_visual
    assert rep.evictions == (w.n_lines - w.budget // w.line_len) * len(sl)


# Random eviction inside the pipeline (score mode 3): integer keys, so scores, evicted sets and
# retained rows must agree with the oracle bit for bit and no near-tie is ever sanctioned.
@pytest.mark.parametrize("w,gpw,n_split,seed", [
    (MID_SPLIT, 0, 0, 1), (MID_SPLIT, 3, 2, 0xFFFFFFFF), (LUMINA_SLICE, 0, 0, 2), (F32_R2, 0, 0, 3), (NO_COND, 1, 0, 4),
    (STREAMING, 0, 0, 5), (F32_WIDE, 0, 0, 6), (ONE_TOKEN_LINES, 0, 0, 7), (NO_ANCHOR_R3, 2, 2, 8),
], ids=lambda x: getattr(x, "name", str(x)))
def test_random_eviction_every_slice(w, gpw, n_split, seed):
    rep = run_parity(w, all_slices(w), groups_per_wave=gpw, n_split=n_split, score_mode=3, random_seed=seed)
    say(f"{w.name} random eviction seed {seed}: {rep}")
    assert rep.steps == w.n_visual and rep.sanctioned == 0 and rep.max_score_rel == 0.0


@pytest.mark.parametrize("w", [synth.LLAMAGEN_XL, synth.LUMINA_768], ids=lambda w: w.name)
def test_full_size_random_eviction_sampled_slices(w):
    sl = _sample(w, n_heads=4 if w is synth.LLAMAGEN_XL else 1)
    rep = run_parity(w, sl, score_mode=3, random_seed=20251204, layers_call=True,
                     progress=say if w.n_lines > 30 else None)
    say(f"{w.name} random eviction: {len(sl)} slices: {rep}")
    assert rep.steps == w.n_visual and rep.sanctioned == 0 and rep.max_score_rel == 0.0
    assert rep.evictions == (w.n_lines - w.budget // w.line_len) * len(sl)


def test_full_size_accumulated_attention_sampled_slices():
    w = synth.LLAMAGEN_XL
    rep = run_parity(w, _sample(w, n_heads=2), score_mode=2, layers_call=True)
    say(f"{w.name} mode 2: {rep}")
    assert rep.steps == w.n_visual and rep.evictions == 20 * len(_sample(w, n_heads=2))


@pytest.mark.parametrize("w", [synth.LLAMAGEN_XL, synth.JANUS_PRO_1B, synth.JANUS_PRO_7B], ids=lambda w: w.name)
def test_full_size_full_cache_sampled_slices(w):
    """The full-cache leg of the benchmark (B = N, the speed-up's denominator): whole images."""
    wf = w.full_cache()
    sl = _sample(wf, n_heads=4)
    rep = run_parity(wf, sl, layers_call=True)
    say(f"{wf.name}: {len(sl)} slices: {rep}")
    assert rep.steps == w.n_visual and rep.evictions == 0


def test_lumina_full_cache_whole_image():
    """Full-cache Lumina shape (T grows to 256 + 2352 keys): the whole image, so that every split
    count the planner reaches (1 .. 6 workgroups per pair) and the merge kernel at each of them is
    compared with the oracle; two slices (4 s of oracle time each)."""
    wf = synth.LUMINA_768.full_cache()
    cfg = binding.cfg_from_workload(wf)
    splits = {binding.linear_plan_shape(cfg, t)["n_split"] for t in range(wf.n_cond, wf.n_cond + wf.n_visual)}
    assert splits == {1, 2, 3, 4, 5, 6}
    rep = run_parity(wf, sampled_slices(wf, [wf.n_layers - 1], [wf.batch - 1], [0, 17]), progress=say,
                     layers_call=True)
    say(f"{wf.name}: {rep}")
    assert rep.steps == wf.n_visual and rep.evictions == 0


def test_state_machine_errors():
    w = synth.shrink(synth.TINY_B, n_heads=2)
    cfg = binding.cfg_from_workload(w)
    cache = binding.LineARCache(cfg)
    kc, vc = synth.cond_kv(w, "cuda:0")
    cache.start_image(kc, vc)
    q, k, v = synth.step_qkv(w, 0, "cuda:0")
    out = torch.empty((w.batch, w.n_heads, w.head_dim), dtype=torch.float32, device="cuda:0")
    with pytest.raises(binding.LinearError) as e:
        cache.end_of_line_evict(0)                       # middle (start) of a line
    assert e.value.code == binding.LINEAR_ESTATE
    with pytest.raises(binding.LinearError) as e:
        cache.decode_step(1, q[0], k[0], v[0], out)      # layer out of range
    assert e.value.code == binding.LINEAR_EINVAL
    with pytest.raises(binding.LinearError) as e:
        cache.scores(0)                                  # line 1 does not evict
    assert e.value.code == binding.LINEAR_ESTATE
    for i in range(w.line_len):
        cache.decode_step(0, q[0], k[0], v[0], out)
    assert binding.kv_length(cache.handle, 0) == (w.n_cond + w.line_len, w.line_len, 0)
    with pytest.raises(binding.LinearError) as e:
        cache.decode_step(0, q[0], k[0], v[0], out)      # line complete, eviction due
    assert e.value.code == binding.LINEAR_ESTATE
    assert binding.kv_length(cache.handle, 0) == (w.n_cond + w.line_len, w.line_len, 0)
    with pytest.raises(binding.LinearError) as e:
        binding.decode_step(cache.handle, 0, q[0].data_ptr() + 2, k[0].data_ptr(), v[0].data_ptr(),
                            out.data_ptr())
    assert e.value.code == binding.LINEAR_EALIGN
    cache.end_of_line_evict(0)
    for line in range(1, w.n_lines):
        for i in range(w.line_len):
            cache.decode_step(0, q[0], k[0], v[0], out)
        cache.end_of_line_evict(0)
    with pytest.raises(binding.LinearError) as e:
        cache.decode_step(0, q[0], k[0], v[0], out)      # image complete
    assert e.value.code == binding.LINEAR_ESTATE
    with pytest.raises(binding.LinearError):
        binding.linear_set_tuning(cache.handle, 17, 0)
    with pytest.raises(binding.LinearError):
        binding.linear_set_tuning(cache.handle, 0, 65)
    torch.cuda.synchronize()
    cache.close()


def test_repeatable_bit_for_bit():
    """Two runs of the same image give identical outputs, scores and retained sets
    (in-place compaction and the split merge have no order-dependent result)."""
    w = LUMINA_SLICE
    dev = "cuda:0"
    results = []
    for _ in range(2):
        cache = binding.LineARCache(binding.cfg_from_workload(w))
        kc, vc = synth.cond_kv(w, dev)
        cache.start_image(kc, vc)
        outs = []
        out = torch.empty((w.n_layers, w.batch, w.n_heads, w.head_dim), dtype=torch.float32, device=dev)
        for step in range(w.n_visual):
            q, k, v = synth.step_qkv(w, step, dev)
            cache.decode_step(0, q[0], k[0], v[0], out[0])
            outs.append(out.clone())
            if (step + 1) % w.line_len == 0:
                cache.end_of_line_evict(0)
        kg, vg, pg = cache.gather(0)
        results.append((torch.stack(outs), kg.clone(), vg.clone(), pg.clone()))
        cache.close()
    for a, b in zip(*results):
        assert torch.equal(a, b)


@pytest.mark.parametrize("guide_queue", [binding.LINEAR_QUEUE_LOGITS, binding.LINEAR_QUEUE_QUERIES], ids=["logits", "queries"])
def test_scores_in_mid_line_and_gather_options(guide_queue):
    """kv_scores before the line is complete returns the partial sum of Eq. 9 over the queries
    queued so far (still divided by n); kv_gather accepts NULL outputs."""
    import numpy as np
    from parity_harness import oracle

    o = oracle()
    w = synth.shrink(synth.TINY_C, n_heads=2)
    dev = "cuda:0"
    cache = binding.LineARCache(binding.cfg_from_workload(w, guide_queue=guide_queue))
    kc, vc = synth.cond_kv(w, dev)
    cache.start_image(kc, vc)
    out = torch.empty((w.batch, w.n_heads, w.head_dim), dtype=torch.float32, device=dev)
    f64 = lambda t: t.to(torch.float64).cpu().numpy()
    sl = [o.CacheSlice(f64(kc[0, 0, h]), f64(vc[0, 0, h]), line_len=w.line_len, n_lines=w.n_lines,
                       budget=w.budget, n_init=w.n_init, n_recent_lines=w.n_recent_lines) for h in range(2)]
    first_evicting_step = (w.budget // w.line_len - 1) * w.line_len
    for step in range(first_evicting_step + 5):
        q, k, v = synth.step_qkv(w, step, dev)
        cache.decode_step(0, q[0], k[0], v[0], out)
        for h in range(2):
            sl[h].step(f64(q[0, 0, h]), f64(k[0, 0, h]), f64(v[0, 0, h]))
        if (step + 1) % w.line_len == 0:
            cache.end_of_line_evict(0)
            for h in range(2):
                sl[h].end_of_line()
    got = cache.scores(0).cpu().numpy()             # 5 of 8 queries queued
    for h in range(2):
        lo, hi = sl[h].mid_range()
        ref = o.saliency(np.stack(sl[h].guide_q), np.stack(sl[h].K[lo:hi]), sl[h].scale) * 5 / w.line_len
        np.testing.assert_allclose(got[0, h], ref, rtol=1e-4, atol=1e-7)
    n = binding.kv_gather(cache.handle, 0, 0, 0, 0)   # all outputs NULL: only the length
    assert n == binding.kv_length(cache.handle, 0)[0] == w.n_cond + first_evicting_step + 5
    pos = torch.empty((w.batch, w.n_heads, n), dtype=torch.int32, device=dev)
    assert binding.kv_gather(cache.handle, 0, 0, 0, pos.data_ptr()) == n
    assert pos[0, 0].tolist() == sl[0].pos
    cache.close()


def test_gather_then_resume_in_a_new_handle():
    """Export of the retained cache and restart from it: a new handle primed with the gathered
    rows as its conditional prefix continues with the same attention outputs (the exported
    rows are exactly what the next steps attend to)."""
    w = synth.Workload("resume", 1, 2, 3, 64, 4, 8, 8, 24, 4, 1, "bf16", 31)
    dev = "cuda:0"
    a = binding.LineARCache(binding.cfg_from_workload(w))
    kc, vc = synth.cond_kv(w, dev)
    a.start_image(kc, vc)
    out = torch.empty((w.batch, w.n_heads, w.head_dim), dtype=torch.float32, device=dev)
    stop = 5 * w.line_len                       # two evictions done
    for step in range(stop):
        q, k, v = synth.step_qkv(w, step, dev)
        a.decode_step(0, q[0], k[0], v[0], out)
        if (step + 1) % w.line_len == 0:
            a.end_of_line_evict(0)
    kg, vg, pg = a.gather(0)
    assert kg.shape[2] == w.n_cond + w.budget - w.line_len
    # continue in the original handle and, in parallel, in a full-cache handle whose prefix is
    # the exported cache: until the next eviction both see the same keys.
    w2 = synth.Workload("resume-b", 1, 2, 3, 64, kg.shape[2], 8, 1, 8, 0, 1, "bf16", 31)
    b = binding.LineARCache(binding.cfg_from_workload(w2))
    b.start_image(kg[None], vg[None])
    out_b = torch.empty_like(out)
    for step in range(stop, stop + w.line_len):
        q, k, v = synth.step_qkv(w, step, dev)
        a.decode_step(0, q[0], k[0], v[0], out)
        b.decode_step(0, q[0], k[0], v[0], out_b)
        assert torch.allclose(out, out_b, atol=2e-6, rtol=0), f"step {step}"
    a.close()
    b.close()


def test_layers_entry_points_report_errors():
    w = synth.shrink(synth.TINY_B, n_heads=2)
    w = synth.Workload("two-layers", 2, 1, 2, 64, 8, 8, 8, 24, 4, 1, "f32", 32)
    dev = "cuda:0"
    cache = binding.LineARCache(binding.cfg_from_workload(w))
    kc, vc = synth.cond_kv(w, dev)
    cache.start_image(kc, vc)
    q, k, v = synth.step_qkv(w, 0, dev)
    out = torch.empty((w.n_layers, w.batch, w.n_heads, w.head_dim), dtype=torch.float32, device=dev)
    stride, ostride = q[0].numel() * 4, out[0].numel() * 4
    args = (q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr())
    with pytest.raises(binding.LinearError) as e:
        binding.decode_step_layers(cache.handle, 1, 2, *args, stride, ostride)     # runs past the last layer
    assert e.value.code == binding.LINEAR_EINVAL
    with pytest.raises(binding.LinearError) as e:
        binding.decode_step_layers(cache.handle, 0, 2, *args, stride + 4, ostride)  # stride not a multiple of 16
    assert e.value.code == binding.LINEAR_EALIGN
    with pytest.raises(binding.LinearError) as e:
        binding.end_of_line_evict_layers(cache.handle, 0, 2)                      # line not complete
    assert e.value.code == binding.LINEAR_ESTATE
    assert binding.kv_length(cache.handle, 0) == (w.n_cond, 0, 0)
    binding.decode_step_layers(cache.handle, 0, 0, *args, stride, ostride)         # count 0: nothing
    for _ in range(w.line_len):
        binding.decode_step_layers(cache.handle, 0, 2, *args, stride, ostride)
    binding.end_of_line_evict_layers(cache.handle, 0, 2)
    assert binding.kv_length(cache.handle, 1) == (w.n_cond + w.line_len, 0, 1)
    torch.cuda.synchronize()
    cache.close()


@pytest.mark.parametrize("guide_queue", [binding.LINEAR_QUEUE_LOGITS, binding.LINEAR_QUEUE_QUERIES], ids=["logits", "queries"])
@pytest.mark.parametrize("n,budget,lines", [(8, 1608, 203), (8, 1672, 211), (24, 2088, 89)],
                         ids=["queue-51KB", "queue-73KB", "queue-196KB"])
def test_largest_mid_regions(n, budget, lines, guide_queue):
    """Mid regions of 1600 and 1664 candidates at n = 8 (their line's logits fit the 64 KiB of
    LDS every device grants, resp. only the 160 KiB of this one) and of 2040 candidates at
    n = 24 (196 KB: read from global memory instead), with the keys split over several
    workgroups: two evictions each, oracle on both heads."""
    w = synth.Workload("largest-mid", 1, 1, 2, 64, 5, n, lines, budget, n if n > 8 else 0, 1, "bf16", 33)
    rep = run_parity(w, all_slices(w), progress=None, guide_queue=guide_queue)
    say(f"{w.name} n={n} B={budget} queue {guide_queue}: {rep}")
    assert rep.evictions == 2 * 2 and rep.steps == w.n_visual
    with pytest.raises(binding.LinearError):      # more than 2048 candidates are refused
        binding.linear_workspace_bytes(binding.cfg_from_workload(
            synth.Workload("too-large-mid", 1, 1, 2, 64, 5, 8, 400, 2072, 0, 1, "bf16", 33)))


def test_lumina_1024_shape_sampled_slices():
    """The paper's largest model shape (N = 4160, rho = 1/8; not one of the five benchmark
    workloads): 520-key budget, 390 candidates per eviction, 56 evictions; its guide queue
    (65 x 392 floats) does not fit LDS."""
    w = synth.LUMINA_1024
    sl = sampled_slices(w, [0, w.n_layers - 1], [w.batch - 1], [0, 13, 31])
    rep = run_parity(w, sl, progress=say, layers_call=True)
    say(f"{w.name}: {rep}")
    assert rep.steps == w.n_visual and rep.evictions == 56 * len(sl)


@pytest.mark.parametrize("w", [synth.LLAMAGEN_XL, synth.JANUS_PRO_1B], ids=lambda w: w.name)
def test_full_size_properties_every_pair(w):
    """What holds for every (layer, sequence, head) of a full-size image, checked on all of them
    with library routines (the oracle only replays sampled slices): retained positions ascend,
    contain the prefix, the anchor and the recent lines, and shrink monotonically (an evicted
    token never returns); retained K/V rows are bit-identical copies of the inputs at those
    positions; each attention output equals softmax(q K^T / sqrt(d)) V over the rows the cache
    held at that step (torch, fp32), at the last step of several lines."""
    dev = "cuda:0"
    cache = binding.LineARCache(binding.cfg_from_workload(w), dev)
    kc, vc = synth.cond_kv(w, dev)
    cache.start_image(kc, vc)
    qs, ks, vs = synth.image_qkv(w, dev)                       # [N, L, Bz, H, d]
    out = torch.empty((w.n_layers, w.batch, w.n_heads, w.head_dim), dtype=torch.float32, device=dev)
    n, C, B = w.line_len, w.n_cond, w.budget
    stride, ostride = qs[0, 0].numel() * qs.element_size(), out[0].numel() * 4
    check_lines = {1, B // n, B // n + 1, w.n_lines // 2, w.n_lines}
    layers = sorted({0, w.n_layers // 2, w.n_layers - 1})
    prev = {l: None for l in layers}
    scale = 1.0 / w.head_dim ** 0.5
    for step in range(w.n_visual):
        line = step // n + 1
        last_of_line = (step + 1) % n == 0
        before = None
        if last_of_line and line in check_lines:
            # cache rows before the step; the step then appends its own k, v
            before = {l: cache.gather(l) for l in layers}
        binding.decode_step_layers(cache.handle, 0, w.n_layers, qs[step].data_ptr(), ks[step].data_ptr(),
                                   vs[step].data_ptr(), out.data_ptr(), stride, ostride, cache.stream())
        if before is not None:
            for l in layers:
                kg, vg, _ = before[l]
                K = torch.cat((kg.float(), ks[step, l].float().unsqueeze(2)), dim=2)      # [Bz, H, T, d]
                V = torch.cat((vg.float(), vs[step, l].float().unsqueeze(2)), dim=2)
                logits = torch.einsum("bhd,bhtd->bht", qs[step, l].float(), K) * scale
                ref = torch.einsum("bht,bhtd->bhd", torch.softmax(logits, dim=-1), V)
                err = (out[l] - ref).abs().max().item()
                assert err <= 2e-4, f"{w.name}: output differs by {err:.3e} at step {step} layer {l}"
        if not last_of_line:
            continue
        binding.end_of_line_evict_layers(cache.handle, 0, w.n_layers, cache.stream())
        for l in layers:
            kg, vg, pg = cache.gather(l)                       # [Bz, H, T, d], [Bz, H, T]
            T = pg.shape[-1]
            evicted = B // n <= line <= w.n_lines - 1
            assert T == C + (B - n if evicted else min(line * n, B))
            pos = pg.long()
            assert bool((pos[..., 1:] > pos[..., :-1]).all())
            head = C + min(w.n_init, line * n)
            assert bool((pos[..., :head] == torch.arange(head, device=dev)).all())
            tail = min(w.n_recent_lines * n, line * n)
            newest = C + line * n - 1
            assert bool((pos[..., T - tail:] == torch.arange(newest - tail + 1, newest + 1, device=dev)).all())
            if prev[l] is not None:
                # every retained position was retained after the previous line or belongs to this line
                was = torch.zeros((w.batch, w.n_heads, C + w.n_visual), dtype=torch.bool, device=dev)
                was.scatter_(2, prev[l], True)
                was[..., C + (line - 1) * n: C + line * n] = True
                assert bool(was.gather(2, pos).all())
            prev[l] = pos
            # rows are copies of the inputs at their positions
            vis = pos[..., C:] - C                              # [Bz, H, T - C] step index of each visual row
            kin = ks[:, l].permute(1, 2, 0, 3)                  # [Bz, H, N, d]
            vin = vs[:, l].permute(1, 2, 0, 3)
            idx = vis.unsqueeze(-1).expand(-1, -1, -1, w.head_dim)
            assert torch.equal(kg[..., C:, :], kin.gather(2, idx))
            assert torch.equal(vg[..., C:, :], vin.gather(2, idx))
            assert torch.equal(kg[..., :C, :], kc[l]) and torch.equal(vg[..., :C, :], vc[l])
    torch.cuda.synchronize()
    cache.close()


def test_more_layers_than_one_end_of_line_launch_covers():
    """50 layers: end_of_line_evict_layers needs two launches (48 + 2 layers); the oracle follows
    layers on both sides of the boundary."""
    w = synth.Workload("many-layers", 50, 1, 2, 64, 3, 4, 7, 12, 4, 1, "bf16", 34)
    sl = sampled_slices(w, [0, 47, 48, 49], [0], [0, 1])
    rep = run_parity(w, sl, layers_call=True)
    say(f"{w.name}: {rep}")
    assert rep.steps == w.n_visual and rep.evictions == (7 - 3 - 1 + 1) * len(sl)


def test_decode_steps_replayed_from_a_hip_graph():
    """The decode steps of a line captured into a HIP graph (the launch sequence is static: cache
    lengths do not depend on the data) and replayed give, on every replay, what the same calls
    give when enqueued directly; eager work and synchronisations sit between the replays.  The
    library enqueues kernels only (no memset, no allocation), so every call can be captured."""
    w = MID_SPLIT
    dev = "cuda:0"
    kc, vc = synth.cond_kv(w, dev)
    n, L = w.line_len, w.n_layers
    lines = w.budget // n + 1                                     # up to and including two evicting lines
    qs, ks, vs = synth.image_qkv(w, dev, steps=lines * n)
    stride = qs[0, 0].numel() * qs.element_size()

    def run(use_graph):
        cache = binding.LineARCache(binding.cfg_from_workload(w), dev)
        cache.start_image(kc, vc)
        outs = torch.zeros((lines * n, L, w.batch, w.n_heads, w.head_dim), dtype=torch.float32, device=dev)
        ostride = outs[0, 0].numel() * 4
        for line in range(lines):
            def steps(stream):
                for s in range(line * n, (line + 1) * n):
                    binding.decode_step_layers(cache.handle, 0, L, qs[s].data_ptr(), ks[s].data_ptr(),
                                               vs[s].data_ptr(), outs[s].data_ptr(), stride, ostride, stream)
            if use_graph:
                torch.cuda.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    steps(torch.cuda.current_stream().cuda_stream)
                first = None
                for _ in range(3):
                    outs[line * n:(line + 1) * n].zero_()           # eager work between the replays
                    g.replay()
                    torch.cuda.synchronize()
                    got = outs[line * n:(line + 1) * n].clone()
                    assert first is None or torch.equal(got, first)
                    first = got
            else:
                steps(cache.stream())
            binding.end_of_line_evict_layers(cache.handle, 0, L, cache.stream())
        torch.cuda.synchronize()
        kept = [tuple(t.clone() for t in cache.gather(l)) for l in range(L)]
        cache.close()
        return outs, kept

    eager_out, eager_kept = run(False)
    graph_out, graph_kept = run(True)
    assert torch.equal(graph_out, eager_out)
    for a, b in zip(eager_kept, graph_kept):
        for x, y in zip(a, b):
            assert torch.equal(x, y)


def test_table4_batch_of_512_sequences():
    """The batch of the paper's efficiency table for the N = 576 class-conditional model (256 images,
    both guidance halves = 512 sequences, 10240 pairs per launch): other launch plans than the
    64-sequence benchmark; oracle on eight slices spread over the batch."""
    from dataclasses import replace
    w = replace(synth.LLAMAGEN_XL, batch=512, name="llamagen-xl-seq512")
    sl = sampled_slices(w, [0, w.n_layers - 1], [0, 255, 511], [0, 19]) + [(17, 300, 7), (17, 77, 11)]
    rep = run_parity(w, sl, layers_call=True)
    say(f"{w.name}: {len(sl)} slices: {rep}")
    assert rep.steps == w.n_visual and rep.evictions == 20 * len(sl)


def test_measurement_aids_run_and_check_their_arguments():
    """linear_probe_stream / linear_probe_empty only read: a buffer they stream over is unchanged,
    and bad arguments come back as error codes."""
    dev = "cuda:0"
    g = torch.Generator(device=dev).manual_seed(3)
    bufs = [torch.randint(0, 255, (6 * 40 * 256,), dtype=torch.uint8, device=dev, generator=g) for _ in range(4)]
    before = [b.clone() for b in bufs]
    kp, vp = [bufs[0].data_ptr(), bufs[1].data_ptr()], [bufs[2].data_ptr(), bufs[3].data_ptr()]
    binding.linear_probe_stream(kp, vp, 6, 33, 40, 256)
    binding.linear_probe_stream(kp, vp, 6, 40, 40, 256)
    binding.linear_probe_empty(3, 6, 64)
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(bufs, before))
    for bad in (dict(rows=41), dict(rows=0), dict(row_bytes=24), dict(n_pairs=0)):
        kw = dict(n_pairs=6, rows=33, pitch_rows=40, row_bytes=256)
        kw.update(bad)
        with pytest.raises(binding.LinearError) as e:
            binding.linear_probe_stream(kp, vp, **kw)
        assert e.value.code == binding.LINEAR_EINVAL
    with pytest.raises(binding.LinearError):
        binding.linear_probe_empty(1, 0, 64)
    with pytest.raises(binding.LinearError):
        binding.linear_probe_empty(1, 1, 2048)
