"""Pins of the input generator's rotary embedding (synth.rope, synth.rope_cos_sin), which is the
reference of the fused rotation in decode_step_rope: what the mathematics of a rotation fixes,
computed here with the math module and by hand, not by calling the generator on itself."""
import math

import pytest
import torch

from paper_2512_04857_amd import synth


def test_position_zero_is_the_identity():
    x = torch.randn(3, 5, 1, 64, generator=torch.Generator().manual_seed(1))
    assert torch.equal(synth.rope(x, torch.tensor([0])), x)
    cs = synth.rope_cos_sin(synth.LLAMAGEN_XL, 0)
    assert torch.equal(cs[:32], torch.ones(32)) and torch.equal(cs[32:], torch.zeros(32))


@pytest.mark.parametrize("d", [2, 4, 64, 128])
def test_every_pair_keeps_its_norm(d):
    x = torch.randn(7, 4, d, generator=torch.Generator().manual_seed(2), dtype=torch.float32)
    y = synth.rope(x, torch.tensor([0, 1, 17, 640]))
    half = d // 2
    before = x[..., :half] ** 2 + x[..., half:] ** 2          # element t is paired with t + d/2
    after = y[..., :half] ** 2 + y[..., half:] ** 2
    torch.testing.assert_close(after, before, rtol=2e-6, atol=1e-6)


def test_two_dimensions_rotate_by_the_position_itself():
    """d = 2: one pair, angle = position * theta^0 = position radians, whatever theta is."""
    for p in (1, 2, 3, 10):
        y = synth.rope(torch.tensor([[1.0, 0.0]]), torch.tensor([p]))
        assert abs(y[0, 0].item() - math.cos(p)) < 1e-6 and abs(y[0, 1].item() - math.sin(p)) < 1e-6
        y = synth.rope(torch.tensor([[0.0, 1.0]]), torch.tensor([p]))
        assert abs(y[0, 0].item() + math.sin(p)) < 1e-6 and abs(y[0, 1].item() - math.cos(p)) < 1e-6


def test_hand_worked_four_dimensions():
    """d = 4, theta = 1e4, position 2: pair (x0, x2) turns by 2 rad, pair (x1, x3) by
    2 * 1e4^(-2/4) = 0.02 rad; x = (1, 2, 3, 4)."""
    y = synth.rope(torch.tensor([[1.0, 2.0, 3.0, 4.0]]), torch.tensor([2]))[0].tolist()
    want = [1 * math.cos(2) - 3 * math.sin(2), 2 * math.cos(0.02) - 4 * math.sin(0.02),
            1 * math.sin(2) + 3 * math.cos(2), 2 * math.sin(0.02) + 4 * math.cos(0.02)]
    assert max(abs(a - b) for a, b in zip(y, want)) < 1e-6


def test_rotations_compose_and_logits_depend_on_the_distance_only():
    g = torch.Generator().manual_seed(3)
    q, k = torch.randn(1, 64, generator=g), torch.randn(1, 64, generator=g)
    twice = synth.rope(synth.rope(q, torch.tensor([5])), torch.tensor([9]))
    torch.testing.assert_close(twice, synth.rope(q, torch.tensor([14])), rtol=1e-5, atol=1e-5)
    a = (synth.rope(q, torch.tensor([5])) * synth.rope(k, torch.tensor([3]))).sum()
    b = (synth.rope(q, torch.tensor([112])) * synth.rope(k, torch.tensor([110]))).sum()
    assert abs(a.item() - b.item()) < 1e-4


@pytest.mark.parametrize("w", [synth.TINY_B, synth.JANUS_PRO_7B], ids=lambda w: w.name)
def test_table_row_holds_the_cosines_then_the_sines_of_the_pair_angles(w):
    d, p = w.head_dim, w.n_cond + 37
    cs = synth.rope_cos_sin(w, p).tolist()
    assert len(cs) == d
    for t in (0, 1, d // 4, d // 2 - 1):
        ang = p * 1.0e4 ** (-2.0 * t / d)
        assert abs(cs[t] - math.cos(ang)) < 1e-6 and abs(cs[d // 2 + t] - math.sin(ang)) < 1e-6
    # the row is what the generator itself multiplies by: rotating a basis vector reads it back
    e = torch.zeros(1, d)
    e[0, 3] = 1.0
    y = synth.rope(e, torch.tensor([p]))[0]
    assert abs(y[3].item() - cs[3]) < 1e-7 and abs(y[d // 2 + 3].item() - cs[d // 2 + 3]) < 1e-7


def test_unrotated_draw_and_its_rotation_are_the_same_tokens():
    """step_qkv_unrotated hands out the storage-rounded draw and an fp32 rotation of exactly
    those rounded values; v is untouched by the rotation."""
    w = synth.shrink(synth.JANUS_PRO_1B, n_layers=1, batch=1, n_heads=2)
    q, k, v, q_rot, k_rot = synth.step_qkv_unrotated(w, 11)
    pos = torch.tensor([w.n_cond + 11])
    assert torch.equal(q_rot, synth.rope(q.float().unsqueeze(-2), pos)[..., 0, :].to(torch.bfloat16))
    assert torch.equal(k_rot, synth.rope(k.float().unsqueeze(-2), pos)[..., 0, :].to(torch.bfloat16))
    n2 = lambda t: (t.float() ** 2).sum(-1)
    torch.testing.assert_close(n2(q_rot), n2(q), rtol=2e-2, atol=0)      # bf16 rounding of a norm-preserving map
    assert torch.equal(v, synth.step_qkv_unrotated(w, 11)[2])
