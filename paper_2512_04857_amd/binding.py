"""ctypes binding of liblinear_kv.so: the same entry points as include/linear_kv.h,
argument marshalling only.  Every step of the path runs in the HIP library; if the
library has not been built this module raises instead of falling back to anything.

`LineARCache` is a convenience holder that lets PyTorch own the device memory (cache,
scratch and I/O tensors) and passes raw pointers and the current stream down.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblinear_kv.so")

LINEAR_OK, LINEAR_EINVAL, LINEAR_ESTATE, LINEAR_ENULL, LINEAR_EALIGN, LINEAR_EHIP, LINEAR_ECAPACITY = 0, -1, -2, -3, -4, -5, -6
LINEAR_F32, LINEAR_BF16 = 0, 1
LINEAR_QUEUE_AUTO, LINEAR_QUEUE_LOGITS, LINEAR_QUEUE_QUERIES = 0, 1, 2
LINEAR_OUT_F32, LINEAR_OUT_ELEM = 0, 1

EXPORTS = ("linear_workspace_bytes", "kv_init", "decode_step", "decode_step_layers",
           "decode_step_rope", "decode_step_rope_layers",
           "end_of_line_evict", "end_of_line_evict_layers", "kv_scores",
           "decode_step_static", "linear_static_scratch_bytes", "linear_probe_stream", "linear_probe_empty",
           "kv_gather", "kv_length", "linear_set_tuning", "linear_plan_shape", "kv_free", "linear_strerror",
           "linear_last_hip_error")


class LinearCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "batch", "n_heads", "head_dim", "n_cond", "line_len", "n_lines", "budget",
        "n_init", "n_recent_lines", "dtype", "score_mode", "guide_queue")] + [("scale", C.c_float), ("seed", C.c_uint32), ("out_dtype", C.c_int32)]


class LinearError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        msg = lib().linear_strerror(code).decode()
        if code == LINEAR_EHIP:
            msg += f" (hipError {lib().linear_last_hip_error()})"
        super().__init__(f"{what}: {msg} [{code}]")


_lib = None


def lib() -> C.CDLL:
    """The loaded library; built by `python -m paper_2512_04857_amd.build` or
    __graft_entry__.build()."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build the HIP library first "
                "(python -m paper_2512_04857_amd.build); there is no fallback path")
        L = C.CDLL(LIB_PATH)
        vp, i32 = C.c_void_p, C.c_int32
        L.linear_workspace_bytes.argtypes = [C.POINTER(LinearCfg), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.kv_init.argtypes = [C.POINTER(LinearCfg), C.POINTER(vp), C.POINTER(vp), vp, C.POINTER(vp),
                              C.POINTER(vp), vp, C.POINTER(vp)]
        L.decode_step.argtypes = [vp, i32, vp, vp, vp, vp, vp]
        L.decode_step_layers.argtypes = [vp, i32, i32, vp, vp, vp, vp, C.c_size_t, C.c_size_t, vp]
        L.decode_step_rope.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp]
        L.decode_step_rope_layers.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, C.c_size_t, C.c_size_t, vp]
        L.end_of_line_evict.argtypes = [vp, i32, vp]
        L.end_of_line_evict_layers.argtypes = [vp, i32, i32, vp]
        L.kv_scores.argtypes = [vp, i32, vp, C.POINTER(i32), vp]
        L.kv_gather.argtypes = [vp, i32, vp, vp, vp, C.POINTER(i32), vp]
        L.kv_length.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
        L.linear_set_tuning.argtypes = [vp, i32, i32]
        L.linear_plan_shape.argtypes = [C.POINTER(LinearCfg), i32, i32, i32, C.POINTER(i32)]
        L.kv_free.argtypes = [vp]
        L.decode_step_static.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, C.c_float, i32, vp, vp]
        L.linear_static_scratch_bytes.argtypes = [C.POINTER(C.c_size_t)]
        L.linear_probe_stream.argtypes = [C.POINTER(vp), C.POINTER(vp), i32, i32, i32, i32, i32, vp]
        L.linear_probe_empty.argtypes = [i32, i32, i32, vp]
        L.linear_strerror.argtypes = [C.c_int]
        L.linear_strerror.restype = C.c_char_p
        L.linear_last_hip_error.argtypes = []
        for name in EXPORTS:
            if name != "linear_strerror":
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(code: int, what: str) -> None:
    if code != LINEAR_OK:
        raise LinearError(code, what)


def make_cfg(*, n_layers, batch, n_heads, head_dim, n_cond, line_len, n_lines, budget, n_init,
             n_recent_lines, dtype, score_mode=0, guide_queue=0, scale=0.0, seed=0, out_dtype=0) -> LinearCfg:
    dt = {"f32": LINEAR_F32, "bf16": LINEAR_BF16}.get(dtype, dtype)
    return LinearCfg(n_layers, batch, n_heads, head_dim, n_cond, line_len, n_lines, budget, n_init,
                     n_recent_lines, dt, score_mode, guide_queue, scale, seed, out_dtype)


def cfg_from_workload(w, score_mode=0, guide_queue=0, scale=0.0, seed=0, out_dtype=0) -> LinearCfg:
    return make_cfg(n_layers=w.n_layers, batch=w.batch, n_heads=w.n_heads, head_dim=w.head_dim,
                    n_cond=w.n_cond, line_len=w.line_len, n_lines=w.n_lines, budget=w.budget,
                    n_init=w.n_init, n_recent_lines=w.n_recent_lines, dtype=w.dtype,
                    score_mode=score_mode, guide_queue=guide_queue, scale=scale, seed=seed, out_dtype=out_dtype)


# ------------------------------------------------------------- thin wrappers ---
def linear_workspace_bytes(cfg: LinearCfg) -> tuple[int, int]:
    a, b = C.c_size_t(), C.c_size_t()
    _check(lib().linear_workspace_bytes(C.byref(cfg), C.byref(a), C.byref(b)), "linear_workspace_bytes")
    return a.value, b.value


def _ptr_array(ptrs):
    if ptrs is None:
        return None
    return (C.c_void_p * len(ptrs))(*ptrs)


def kv_init(cfg: LinearCfg, k_cache, v_cache, scratch: int, k_cond, v_cond, stream: int = 0) -> int:
    h = C.c_void_p()
    _check(lib().kv_init(C.byref(cfg), _ptr_array(k_cache), _ptr_array(v_cache), scratch,
                         _ptr_array(k_cond), _ptr_array(v_cond), stream, C.byref(h)), "kv_init")
    return h.value


def decode_step(kv: int, layer: int, q: int, k: int, v: int, out: int, stream: int = 0) -> None:
    rc = lib().decode_step(kv, layer, q, k, v, out, stream)
    if rc:
        raise LinearError(rc, "decode_step")


def decode_step_layers(kv: int, first_layer: int, count: int, q: int, k: int, v: int, out: int,
                       qkv_stride: int, out_stride: int, stream: int = 0) -> None:
    rc = lib().decode_step_layers(kv, first_layer, count, q, k, v, out, qkv_stride, out_stride, stream)
    if rc:
        raise LinearError(rc, "decode_step_layers")


def decode_step_rope(kv: int, layer: int, q: int, k: int, v: int, cos_sin: int, out: int, stream: int = 0) -> None:
    rc = lib().decode_step_rope(kv, layer, q, k, v, cos_sin, out, stream)
    if rc:
        raise LinearError(rc, "decode_step_rope")


def decode_step_rope_layers(kv: int, first_layer: int, count: int, q: int, k: int, v: int, cos_sin: int,
                            out: int, qkv_stride: int, out_stride: int, stream: int = 0) -> None:
    rc = lib().decode_step_rope_layers(kv, first_layer, count, q, k, v, cos_sin, out, qkv_stride, out_stride,
                                       stream)
    if rc:
        raise LinearError(rc, "decode_step_rope_layers")


def end_of_line_evict_layers(kv: int, first_layer: int, count: int, stream: int = 0) -> None:
    rc = lib().end_of_line_evict_layers(kv, first_layer, count, stream)
    if rc:
        raise LinearError(rc, "end_of_line_evict_layers")


def end_of_line_evict(kv: int, layer: int, stream: int = 0) -> None:
    rc = lib().end_of_line_evict(kv, layer, stream)
    if rc:
        raise LinearError(rc, "end_of_line_evict")


def kv_scores(kv: int, layer: int, out: int, stream: int = 0) -> int:
    m = C.c_int32()
    _check(lib().kv_scores(kv, layer, out, C.byref(m), stream), "kv_scores")
    return m.value


def kv_gather(kv: int, layer: int, k_out: int, v_out: int, pos_out: int, stream: int = 0) -> int:
    n = C.c_int32()
    _check(lib().kv_gather(kv, layer, k_out, v_out, pos_out, C.byref(n), stream), "kv_gather")
    return n.value


def kv_length(kv: int, layer: int) -> tuple[int, int, int]:
    a, b, c = C.c_int32(), C.c_int32(), C.c_int32()
    _check(lib().kv_length(kv, layer, C.byref(a), C.byref(b), C.byref(c)), "kv_length")
    return a.value, b.value, c.value


def linear_set_tuning(kv: int, groups_per_wave: int = 0, n_split: int = 0) -> None:
    _check(lib().linear_set_tuning(kv, groups_per_wave, n_split), "linear_set_tuning")


def linear_plan_shape(cfg: LinearCfg, cached_keys: int, groups_per_wave: int = 0, n_split: int = 0) -> dict:
    out = (C.c_int32 * 6)()
    _check(lib().linear_plan_shape(C.byref(cfg), cached_keys, groups_per_wave, n_split, out), "linear_plan_shape")
    return dict(zip(("n_split", "keys_per_workgroup", "n_waves", "depth", "new_wave", "keys_per_group"), out))


def decode_step_static(dtype: int, head_dim: int, n_pairs: int, cached_keys: int, cache_pitch: int, k_cache: int,
                       v_cache: int, q: int, k: int, v: int, out: int, scale: float = 0.0, n_split: int = 0,
                       stream: int = 0) -> None:
    rc = lib().decode_step_static(dtype, head_dim, n_pairs, cached_keys, cache_pitch, k_cache, v_cache, q, k, v,
                                  scale, n_split, out, stream)
    if rc:
        raise LinearError(rc, "decode_step_static")


def linear_static_scratch_bytes() -> int:
    n = C.c_size_t()
    _check(lib().linear_static_scratch_bytes(C.byref(n)), "linear_static_scratch_bytes")
    return n.value


def linear_probe_stream(k_cache, v_cache, n_pairs: int, rows: int, pitch_rows: int, row_bytes: int,
                        stream: int = 0) -> None:
    _check(lib().linear_probe_stream(_ptr_array(k_cache), _ptr_array(v_cache), len(k_cache), n_pairs, rows,
                                     pitch_rows, row_bytes, stream), "linear_probe_stream")


def linear_probe_empty(launches: int, groups: int, threads: int, stream: int = 0) -> None:
    _check(lib().linear_probe_empty(launches, groups, threads, stream), "linear_probe_empty")


def kv_free(kv: int) -> None:
    _check(lib().kv_free(kv), "kv_free")


# ------------------------------------------------------------ torch plumbing ---
class LineARCache:
    """Device memory (torch tensors) plus a library handle for one image."""

    def __init__(self, cfg: LinearCfg, device="cuda:0"):
        import torch

        self.torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        if self.device.type != "cuda":
            raise RuntimeError("LineARCache needs a GPU device; there is no CPU path")
        cache_bytes, scratch_bytes = linear_workspace_bytes(cfg)
        self.elem = torch.bfloat16 if cfg.dtype == LINEAR_BF16 else torch.float32
        es = 2 if cfg.dtype == LINEAR_BF16 else 4
        self.t_max = cfg.n_cond + cfg.budget
        shape = (cfg.batch, cfg.n_heads, self.t_max, cfg.head_dim)
        assert cache_bytes == cfg.batch * cfg.n_heads * self.t_max * cfg.head_dim * es
        self.k_cache = [torch.empty(shape, dtype=self.elem, device=self.device) for _ in range(cfg.n_layers)]
        self.v_cache = [torch.empty(shape, dtype=self.elem, device=self.device) for _ in range(cfg.n_layers)]
        self.scratch = torch.empty(scratch_bytes, dtype=torch.uint8, device=self.device)
        self.handle = None

    def stream(self) -> int:
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def start_image(self, k_cond=None, v_cond=None):
        """k_cond, v_cond: [L, Bz, H, C, d] tensors (or lists of [Bz, H, C, d])."""
        if self.handle is not None:
            kv_free(self.handle)
            self.handle = None
        kc = vc = None
        if self.cfg.n_cond > 0:
            self._cond = ([k_cond[l].contiguous() for l in range(self.cfg.n_layers)],
                          [v_cond[l].contiguous() for l in range(self.cfg.n_layers)])
            kc = [t.data_ptr() for t in self._cond[0]]
            vc = [t.data_ptr() for t in self._cond[1]]
        self.handle = kv_init(self.cfg, [t.data_ptr() for t in self.k_cache],
                              [t.data_ptr() for t in self.v_cache], self.scratch.data_ptr(), kc, vc,
                              self.stream())

    def decode_step(self, layer, q, k, v, out):
        decode_step(self.handle, layer, q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(),
                    self.stream())

    def end_of_line_evict(self, layer):
        end_of_line_evict(self.handle, layer, self.stream())

    def scores(self, layer):
        c = self.cfg
        mid = c.budget - c.n_init - c.n_recent_lines * c.line_len
        out = self.torch.empty((c.batch, c.n_heads, mid), dtype=self.torch.float32, device=self.device)
        got = kv_scores(self.handle, layer, out.data_ptr(), self.stream())
        assert got == mid
        return out

    def gather(self, layer):
        c = self.cfg
        length = kv_length(self.handle, layer)[0]
        t = self.torch
        k = t.empty((c.batch, c.n_heads, length, c.head_dim), dtype=self.elem, device=self.device)
        v = t.empty_like(k)
        pos = t.empty((c.batch, c.n_heads, length), dtype=t.int32, device=self.device)
        n = kv_gather(self.handle, layer, k.data_ptr(), v.data_ptr(), pos.data_ptr(), self.stream())
        assert n == length
        return k, v, pos

    def close(self):
        if self.handle is not None:
            kv_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:  # noqa: BLE001 - interpreter shutdown
            pass
