"""CPU oracle for the LineAR decode path.  TEST INFRASTRUCTURE, NOT PRODUCT CODE.

A plain, slow, step-by-step transcription of what the paper's method computes
for ONE attention head of ONE sequence in ONE layer (slices never interact):

  * Eq. 2-3   single-query softmax attention over [K_cond, K_visual]
  * Eq. 4     append of the new (k_i, v_i)
  * Sec. 3.3  "Progressive KV Cache Compression Pipeline": no compression while
              fewer than B visual tokens are cached; from then on, at the end of
              every raster line, partition the visual cache into init / mid / rec,
              evict n tokens of mid, keep order (Eq. 5-7)
  * Eq. 8     guide queue: the n queries of the line being generated
  * Eq. 9     saliency S = (1/n) 1^T Softmax(Q_guide K_mid^T / sqrt(d))
  * Eq. 10    E = BottomK(S, n)

Arithmetic is numpy float64 (the paper fixes no precision); inputs are whatever
values the caller passes (the tests pass bf16- or fp32-rounded values upcast).
Nothing here is blocked, fused or reordered, and nothing is shared with the HIP
path: only tests, the smoke check and the benchmark's cpu_baseline leg may
import this module.

Readings of points the paper leaves open are listed in the design notes; the ones
that matter here: conditional tokens are never evicted, never scored and do not
count against B; N_init counts visual tokens; the softmax of Eq. 9 is over the
mid columns only (score_mode 0) -- score_mode 1 instead takes each guide query's
decode-time attention probabilities (softmax over the whole cache) restricted to
mid; score_mode 2 is the paper's "AttAcc" ablation (Sec. 4.4, Table 6: selection by
accumulated attention inside the same pipeline), read the way it describes H2O
(Sec. 4.2: "accumulated attention"): every cached token carries the sum of the
decode-time probabilities it has received from every query since it was appended,
its own included, the sum is never reset and travels with the token; score_mode 3
is random eviction (the paper's Random baseline, Sec. 4.2, Table 3) restricted to
this pipeline's mid region: a candidate's score is a 24-bit integer hash of (seed,
layer, sequence, head, line, original position), so the n evicted tokens are a
reproducible pseudo-random draw that both implementations can compute bit for bit
(the paper's own Random also discards anchor and recent-line tokens, i.e. evicts
outside the partition; that variant is not this pipeline and is not built); the first
eviction happens at the end of line B/n, none after the last line;
BottomK breaks ties by evicting the older (smaller original position) token.

Pins: every function below is pinned by tests/test_oracle_pins.py against
closed forms, library routines, brute force and hand-worked values.  The
*quality* of the heuristic on real images is "parity unpinned": it needs the
paper's trained models and datasets.
"""
from __future__ import annotations

import math

import numpy as np

F = np.float64


def softmax(x: np.ndarray, axis: int = -1) -> np.ndarray:
    """Softmax with the usual max subtraction (a pure rescaling of Eq. 2's
    numerator and denominator)."""
    x = np.asarray(x, dtype=F)
    e = np.exp(x - x.max(axis=axis, keepdims=True))
    return e / e.sum(axis=axis, keepdims=True)


def attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float) -> np.ndarray:
    """Eq. 2: Softmax(q K^T * scale) V for one query q[d], K[T,d], V[T,d]."""
    logits = (np.asarray(K, F) @ np.asarray(q, F)) * scale
    return softmax(logits) @ np.asarray(V, F)


def saliency(Q_guide: np.ndarray, K_mid: np.ndarray, scale: float) -> np.ndarray:
    """Eq. 9: row-wise softmax of Q_guide K_mid^T * scale over the mid tokens,
    then the mean over the n guide queries (the (1/n) 1^T in front)."""
    A = softmax((np.asarray(Q_guide, F) @ np.asarray(K_mid, F).T) * scale, axis=1)
    n = A.shape[0]
    return A.sum(axis=0) / n


def bottom_k(S: np.ndarray, k: int) -> list[int]:
    """Eq. 10: indices of the k least salient entries.  Ties: the entry that
    comes first (the older token) is evicted first.  Returned ascending."""
    order = sorted(range(len(S)), key=lambda j: (S[j], j))
    return sorted(order[:k])


def boundary_gap(S: np.ndarray, k: int) -> float:
    """Relative gap between the largest evicted and the smallest retained score,
    (S_(k+1) - S_(k)) / S_(k+1) on ascending order statistics; inf when nothing
    is retained or nothing evicted."""
    if k <= 0 or k >= len(S):
        return math.inf
    s = np.sort(np.asarray(S, F))
    return float((s[k] - s[k - 1]) / s[k]) if s[k] > 0 else 0.0


M32 = 0xFFFFFFFF


def mix32(x: int) -> int:
    """A 32-bit integer finaliser (two xorshift-multiply rounds and a closing xorshift,
    the published "lowbias32" constants): a bijection of the 32-bit integers."""
    x &= M32
    x ^= x >> 16
    x = (x * 0x7FEB352D) & M32
    x ^= x >> 15
    x = (x * 0x846CA68B) & M32
    x ^= x >> 16
    return x


def random_key(seed: int, layer: int, sequence: int, head: int, line: int, position: int) -> int:
    """score_mode 3: the counter-based pseudo-random score of one candidate at one end of
    line.  The counters are absorbed one by one (add, then mix); the top 24 bits of the
    result are the score, so that it is exactly representable in single precision."""
    h = mix32((seed & M32) ^ 0x9E3779B9)
    for x in (layer, sequence, head, line, position):
        h = mix32((h + x) & M32)
    return h >> 8


class CacheSlice:
    """The visual KV cache of one (layer, sequence, head) under LineAR.

    Entries are kept as python lists of (original position, k row, v row) in
    ascending original position: conditional tokens 0..C-1 first, visual token
    i (1-based) at position C+i-1.
    """

    def __init__(self, K_cond, V_cond, *, line_len, n_lines, budget, n_init,
                 n_recent_lines, scale=None, score_mode=0, seed=0, layer=0, sequence=0, head=0):
        K_cond = np.asarray(K_cond, F)
        V_cond = np.asarray(V_cond, F)
        self.C, self.d = K_cond.shape
        self.n, self.h, self.B = int(line_len), int(n_lines), int(budget)
        self.N = self.n * self.h
        self.N_init, self.r = int(n_init), int(n_recent_lines)
        self.scale = 1.0 / math.sqrt(self.d) if scale is None else float(scale)
        self.score_mode = int(score_mode)
        # score_mode 3 only: the slice's identity, which seeds its random draws
        self.seed, self.layer, self.sequence, self.head = int(seed), int(layer), int(sequence), int(head)
        if self.B % self.n or not (self.n <= self.B <= self.N):
            raise ValueError("budget must be a multiple of the line length within [n, N]")
        self.compresses = self.B < self.N
        if self.compresses and self.N_init + (self.r + 1) * self.n > self.B:
            raise ValueError("N_init + (r+1) n must not exceed B: mid must hold n candidates")
        if self.r < 1 or self.N_init < 0:
            raise ValueError("need r >= 1 and N_init >= 0")
        self.pos = list(range(self.C))
        self.K = [K_cond[j] for j in range(self.C)]
        self.V = [V_cond[j] for j in range(self.C)]
        self.i = 0                   # visual tokens generated so far
        self.guide_q: list[np.ndarray] = []   # Eq. 8 queue (current line's queries)
        self.guide_p: list[np.ndarray] = []   # score_mode 1: their decode probabilities on mid
        self.acc = [0.0] * self.C             # score_mode 2: attention received so far, per entry
        self.pending_eol = False

    # -- bookkeeping the paper states in prose --------------------------------
    @property
    def line(self) -> int:
        """1-based index of the line the most recent token belongs to."""
        return (self.i + self.n - 1) // self.n

    @property
    def visual_len(self) -> int:
        return len(self.pos) - self.C

    def line_evicts(self, line: int) -> bool:
        """Compression is active from the line that fills the budget (line B/n)
        up to the last line but one; nothing is generated after the last line."""
        return self.compresses and self.B // self.n <= line <= self.h - 1

    def mid_range(self) -> tuple[int, int]:
        """Cache index range [lo, hi) of the mid region at the end of an evicting
        line: behind the C conditional and N_init anchor tokens, in front of the r
        most recent lines (the last of which is the line just generated)."""
        lo = self.C + self.N_init
        hi = self.C + self.B - self.r * self.n
        return lo, hi

    # -- Eq. 2-4 --------------------------------------------------------------
    def step(self, q, k, v) -> np.ndarray:
        if self.pending_eol:
            raise RuntimeError("end_of_line() must be called before the next line starts")
        if self.i >= self.N:
            raise RuntimeError("image complete")
        q = np.asarray(q, F)
        self.i += 1
        self.pos.append(self.C + self.i - 1)
        self.K.append(np.asarray(k, F))
        self.V.append(np.asarray(v, F))
        Kmat = np.stack(self.K)
        Vmat = np.stack(self.V)
        logits = (Kmat @ q) * self.scale
        p = softmax(logits)
        out = p @ Vmat
        self.acc.append(0.0)
        if self.score_mode == 2:
            for j in range(len(self.acc)):
                self.acc[j] += float(p[j])
        if self.line_evicts(self.line):
            self.guide_q.append(q)
            lo, hi = self.mid_range()
            self.guide_p.append(p[lo:hi].copy())
        if self.i % self.n == 0:
            self.pending_eol = True
        return out

    # -- Eq. 5-10 ---------------------------------------------------------------
    def scores(self) -> np.ndarray:
        """S^(l) for the line just completed (only meaningful on evicting lines)."""
        lo, hi = self.mid_range()
        if self.score_mode == 0:
            return saliency(np.stack(self.guide_q), np.stack(self.K[lo:hi]), self.scale)
        if self.score_mode == 2:
            return np.asarray(self.acc[lo:hi], dtype=F)
        if self.score_mode == 3:
            return np.asarray([random_key(self.seed, self.layer, self.sequence, self.head, self.line, p)
                               for p in self.pos[lo:hi]], dtype=F)
        return np.stack(self.guide_p).sum(axis=0) / len(self.guide_p)

    def end_of_line(self, force_evict_positions=None) -> dict | None:
        """Synchronisation point at the end of a raster line.  Returns None when
        no compression applies, else a record with the scores, the evicted
        original positions and the boundary gap.  `force_evict_positions`
        overrides the choice (used by the parity harness to re-synchronise after
        a sanctioned near-tie)."""
        if not self.pending_eol:
            raise RuntimeError("end_of_line() in the middle of a line")
        self.pending_eol = False
        line = self.line
        if not self.line_evicts(line):
            self.guide_q, self.guide_p = [], []
            return None
        assert self.visual_len == self.B and len(self.guide_q) == self.n
        lo, hi = self.mid_range()
        S = self.scores()
        chosen = bottom_k(S, self.n)
        evict = [lo + j for j in chosen]
        rec = {
            "line": line,
            "scores": S,
            "mid_positions": list(self.pos[lo:hi]),
            "evicted_positions": [self.pos[j] for j in evict],
            "gap": boundary_gap(S, self.n),
        }
        if force_evict_positions is not None:
            want = set(int(p) for p in force_evict_positions)
            evict = [j for j in range(lo, hi) if self.pos[j] in want]
            if len(evict) != self.n:
                raise ValueError("forced eviction must name n mid tokens")
            rec["forced_positions"] = sorted(want)
        drop = set(evict)
        keep = [j for j in range(len(self.pos)) if j not in drop]
        self.pos = [self.pos[j] for j in keep]
        self.K = [self.K[j] for j in keep]
        self.V = [self.V[j] for j in keep]
        self.acc = [self.acc[j] for j in keep]
        assert self.visual_len == self.B - self.n          # Eq. 6
        self.guide_q, self.guide_p = [], []
        return rec

    def retained(self):
        """(positions, K, V) of the cache in canonical order."""
        return list(self.pos), np.stack(self.K), np.stack(self.V)


def run_slice(K_cond, V_cond, Q, K, V, **cfg):
    """Whole image for one slice.  Q, K, V are [N, d].  Returns the outputs
    [N, d], the list of end-of-line records and the final CacheSlice."""
    sl = CacheSlice(K_cond, V_cond, **cfg)
    outs = np.empty((len(Q), sl.d), dtype=F)
    records = []
    for i in range(len(Q)):
        outs[i] = sl.step(Q[i], K[i], V[i])
        if sl.pending_eol:
            r = sl.end_of_line()
            if r is not None:
                records.append(r)
    return outs, records, sl
