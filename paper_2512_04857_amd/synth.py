"""Seeded synthetic workloads for the LineAR decode path.

This module only *makes inputs*: the shape tables of the five benchmark
workloads and a seeded generator of per-step Q/K/V (iid N(0,1), 1D rotary
position embedding applied to Q and K, rounded to the storage type).  It holds
none of the method's arithmetic (no attention, no scoring, no eviction), so the
CPU oracle's tests and the HIP path's tests can both draw their inputs from it
and be sure they consume bit-identical values.

The synthetic tensors stand in for the activations of trained LlamaGen /
Janus-Pro / Lumina-mGPT models on ImageNet / MS-COCO / GenEval / DPG prompts
(paper Sec. 4.1, "Evaluated Models"): they reproduce the shapes, the prefix
length, the raster-line structure and the storage type, not the attention
statistics of real images.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import torch

ROPE_THETA = 1.0e4
BASE_SEED = 20251204


@dataclass(frozen=True)
class Workload:
    """Shape of one workload.  Symbols follow the paper (Sec. 3.1 and 3.3):
    C conditional tokens, a grid of h lines by n tokens, budget B, anchor length
    N_init and r protected recent lines."""

    name: str
    n_layers: int
    batch: int          # sequences, both classifier-free-guidance halves counted
    n_heads: int
    head_dim: int       # d
    n_cond: int         # C
    line_len: int       # n, tokens per raster line (an end-of-line token counts)
    n_lines: int        # h
    budget: int         # B, a multiple of n; B == h*n keeps the whole cache
    n_init: int         # N_init
    n_recent_lines: int  # r
    dtype: str          # "f32" or "bf16": storage type of Q/K/V and of the cache
    index: int = 0      # offsets the seed so workloads never share a stream

    @property
    def n_visual(self) -> int:
        return self.line_len * self.n_lines

    def full_cache(self) -> "Workload":
        """Same workload with B = N: nothing is ever evicted."""
        return replace(self, name=self.name + "-full", budget=self.n_visual)

    @property
    def torch_dtype(self) -> torch.dtype:
        return {"f32": torch.float32, "bf16": torch.bfloat16}[self.dtype]


def _w(*a, **k) -> Workload:
    return Workload(*a, **k)


# The paper's toy (Fig. 6 caption): 8x8 grid, rho = 3/8.  N_init and r are not
# printed in the paper; three readings are exercised (see the design notes):
#   A  N_init = n, r = 1          -> every candidate is evicted (sink + window)
#   B  N_init = n/2, r = 1        -> 12 candidates, 4 survive
#   C  N_init = n, r = 1, B = 4n  -> 16 candidates, 8 survive
TINY_A = _w("tiny-a", 1, 1, 4, 64, 8, 8, 8, 24, 8, 1, "f32", 1)
TINY_B = _w("tiny-b", 1, 1, 4, 64, 8, 8, 8, 24, 4, 1, "f32", 1)
TINY_C = _w("tiny-c", 1, 1, 4, 64, 8, 8, 8, 32, 8, 1, "f32", 1)
LLAMAGEN_XL = _w("llamagen-xl", 36, 64, 20, 64, 1, 24, 24, 96, 24, 1, "bf16", 2)
JANUS_PRO_1B = _w("janus-pro-1b", 24, 32, 16, 128, 64, 24, 24, 96, 24, 1, "bf16", 3)
JANUS_PRO_7B = _w("janus-pro-7b", 30, 32, 32, 128, 128, 24, 24, 96, 24, 1, "bf16", 4)
LUMINA_768 = _w("lumina-mgpt-768", 32, 8, 32, 128, 256, 49, 48, 294, 49, 1, "bf16", 5)
# Beyond the five benchmark workloads: the paper's largest model (Table 1: N = 4160 = 64 lines of
# 64 tokens + one end-of-line token, rho = 1/8, so B = 520 = 8 lines).
LUMINA_1024 = _w("lumina-mgpt-1024", 32, 8, 32, 128, 256, 65, 64, 520, 65, 1, "bf16", 6)

WORKLOADS = {w.name: w for w in (TINY_A, TINY_B, TINY_C, LLAMAGEN_XL, JANUS_PRO_1B,
                                 JANUS_PRO_7B, LUMINA_768, LUMINA_1024)}


def shrink(w: Workload, *, n_layers=None, batch=None, n_heads=None) -> Workload:
    """A thinner copy (fewer layers / sequences / heads) of a workload.  Slices
    are independent, so a thinner copy is an exact sub-problem."""
    return replace(
        w,
        name=w.name + "-slice",
        n_layers=w.n_layers if n_layers is None else n_layers,
        batch=w.batch if batch is None else batch,
        n_heads=w.n_heads if n_heads is None else n_heads,
    )


def _generator(device, *key: int) -> torch.Generator:
    g = torch.Generator(device=device)
    s = 0x9E3779B97F4A7C15
    for x in key:
        s = (s * 6364136223846793005 + int(x) + 1442695040888963407) % (1 << 63)
    g.manual_seed(s)
    return g


def rope(x: torch.Tensor, positions: torch.Tensor) -> torch.Tensor:
    """Rotary embedding, half-split pairing (x_t, x_{t+d/2}), angle
    p * theta^(-2t/d).  `x` is [..., T, d] fp32, `positions` is [T]."""
    d = x.shape[-1]
    half = d // 2
    t = torch.arange(half, device=x.device, dtype=torch.float64)
    inv = ROPE_THETA ** (-2.0 * t / d)
    ang = positions.to(torch.float64)[:, None] * inv[None, :]
    cos, sin = ang.cos().to(torch.float32), ang.sin().to(torch.float32)
    a, b = x[..., :half], x[..., half:]
    return torch.cat((a * cos - b * sin, a * sin + b * cos), dim=-1)


def cond_kv(w: Workload, device="cpu", seed: int = BASE_SEED):
    """K_cond, V_cond for every layer: two tensors [L, Bz, H, C, d] in the
    workload's storage type (the prefill's result, which the path takes as input)."""
    g = _generator(device, seed, w.index, 0xC0)
    shape = (w.n_layers, w.batch, w.n_heads, w.n_cond, w.head_dim)
    k = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    v = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    k = rope(k, torch.arange(w.n_cond, device=device))
    return k.to(w.torch_dtype).contiguous(), v.to(w.torch_dtype).contiguous()


def step_qkv(w: Workload, step: int, device="cpu", seed: int = BASE_SEED):
    """q, k, v of visual token `step` (0-based) for every layer: three tensors
    [L, Bz, H, d] in the storage type; Q and K rotated at position C + step."""
    g = _generator(device, seed, w.index, 0x51, step)
    shape = (3, w.n_layers, w.batch, w.n_heads, 1, w.head_dim)
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    pos = torch.tensor([w.n_cond + step], device=device)
    q = rope(x[0], pos)[..., 0, :]
    k = rope(x[1], pos)[..., 0, :]
    v = x[2][..., 0, :]
    dt = w.torch_dtype
    return q.to(dt).contiguous(), k.to(dt).contiguous(), v.to(dt).contiguous()


def rope_cos_sin(w: Workload, position: int, device="cpu") -> torch.Tensor:
    """Rotary table row for one absolute position: [d] fp32, the d/2 cosines then the d/2 sines
    of the pair angles position * theta^(-2t/d) (the values `rope` multiplies by)."""
    d = w.head_dim
    t = torch.arange(d // 2, device=device, dtype=torch.float64)
    ang = float(position) * ROPE_THETA ** (-2.0 * t / d)
    return torch.cat((ang.cos(), ang.sin())).to(torch.float32).contiguous()


def step_qkv_unrotated(w: Workload, step: int, device="cpu", seed: int = BASE_SEED):
    """The same draw as step_qkv, handed over the way a model's projection leaves it: q, k, v
    rounded to the storage type and NOT rotated, plus what a rotation in fp32 of those rounded
    values gives, rounded again (q_rot, k_rot) -- the values a consumer that fuses the rotary
    embedding must reproduce.  Returns (q, k, v, q_rot, k_rot), each [L, Bz, H, d]."""
    g = _generator(device, seed, w.index, 0x51, step)
    shape = (3, w.n_layers, w.batch, w.n_heads, 1, w.head_dim)
    dt = w.torch_dtype
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(dt)
    pos = torch.tensor([w.n_cond + step], device=device)
    q_rot = rope(x[0].to(torch.float32), pos).to(dt)[..., 0, :]
    k_rot = rope(x[1].to(torch.float32), pos).to(dt)[..., 0, :]
    return (x[0][..., 0, :].contiguous(), x[1][..., 0, :].contiguous(), x[2][..., 0, :].contiguous(),
            q_rot.contiguous(), k_rot.contiguous())


def image_qkv(w: Workload, device="cpu", seed: int = BASE_SEED, steps: int | None = None):
    """All steps of one image stacked: three tensors [N, L, Bz, H, d]."""
    n = w.n_visual if steps is None else steps
    qs, ks, vs = [], [], []
    for i in range(n):
        q, k, v = step_qkv(w, i, device, seed)
        qs.append(q)
        ks.append(k)
        vs.append(v)
    return torch.stack(qs), torch.stack(ks), torch.stack(vs)
