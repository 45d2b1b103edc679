"""Seeded synthetic inputs for the PicoSpec verification path.

This module only draws random numbers and lays them out; it holds none of the method's
arithmetic (no softmax, no top-k, no acceptance test) and is the one module that both the GPU
path's callers and the CPU oracle's tests use.  The five workloads stand in for the logits the
paper's model pairs would produce on its evaluation prompts: only the vocabulary sizes
(Section 3.3: 128,256 and 151,936), the draft lengths (Section 4.1, Table 4) and the long-tailed
shape of LLM distributions (Section 3.3) are taken from the paper.

Every value is a pure function of (base seed, workload id, tensor id, round, sequence b,
position t), so a subset of sequences can be regenerated alone and equals the full batch.

Layout of one round (what the C-ABI calls expect):
  draft rows   N = sum_b gamma_b, sequence b owns rows seq_off[b] .. seq_off[b+1]-1
  target rows  N + B, sequence b owns rows seq_off[b]+b .. seq_off[b+1]+b (last = bonus position)
  uniforms     [N+B] float32 in [0,1), indexed like target rows
  draft_uniforms [N] float32 in [0,1), one per draft row (drives the edge-side token draw)
bf16 tensors are returned as uint16 bit patterns (round-to-nearest-even of the fp32 values).
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

BASE_SEED = 260319133
_T_TARGET, _T_DRAFT, _T_UNIFORM, _T_DRAFT_UNIFORM, _T_GAMMA = 1, 2, 3, 4, 5


@dataclass(frozen=True)
class Workload:
    name: str
    wid: int
    B: int
    gamma_lo: int
    gamma_hi: int          # gamma_b uniform in [gamma_lo, gamma_hi]; equal => fixed draft length
    V: int
    dtype: str             # "f32" | "bf16"
    T: float
    k: int
    top_p: float           # 0 => plain top-k
    rounds: int
    recipe: str            # "normal3" | "normal4_mix" | "zipf1.1" | "normal5_resample" | "zipf1.2"

    @property
    def gamma_max(self) -> int:
        return self.gamma_hi

    def scaled(self, B: int | None = None, V: int | None = None, k: int | None = None,
               rounds: int | None = None) -> "Workload":
        """Same recipe at a reduced size (for oracle-speed parity tests)."""
        return Workload(self.name + "-scaled", self.wid, B or self.B, self.gamma_lo, self.gamma_hi,
                        V or self.V, self.dtype, self.T, k or self.k, self.top_p,
                        rounds or self.rounds, self.recipe)


WORKLOADS = {
    "cfg1": Workload("cfg1", 1, 1, 4, 4, 32000, "f32", 1.0, 64, 0.0, 1, "normal3"),
    "cfg2": Workload("cfg2", 2, 8, 8, 8, 32000, "bf16", 1.0, 256, 0.0, 1, "normal4_mix"),
    "cfg3": Workload("cfg3", 3, 64, 8, 8, 128256, "bf16", 0.7, 1024, 0.0, 1, "zipf1.1"),
    "cfg4": Workload("cfg4", 4, 256, 16, 16, 151936, "f32", 1.0, 4096, 0.0, 1, "normal5_resample"),
    "cfg5": Workload("cfg5", 5, 512, 1, 16, 152064, "bf16", 1.0, 2048, 0.95, 100, "zipf1.2"),
}


def _rng(*key: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([BASE_SEED, *key])))


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def gammas(w: Workload, rnd: int = 0) -> np.ndarray:
    if w.gamma_lo == w.gamma_hi:
        return np.full(w.B, w.gamma_lo, np.int32)
    return _rng(w.wid, _T_GAMMA, rnd).integers(w.gamma_lo, w.gamma_hi + 1, size=w.B, dtype=np.int32)


def seq_offsets(g: np.ndarray) -> np.ndarray:
    off = np.zeros(g.shape[0] + 1, np.int32)
    np.cumsum(g, out=off[1:])
    return off


def _zipf_row(rng: np.random.Generator, V: int, s: float) -> np.ndarray:
    ranks = rng.permutation(V).astype(np.float32) + np.float32(1.0)
    return (np.float32(-s) * np.log(ranks) + rng.standard_normal(V, dtype=np.float32) * np.float32(0.5))


def target_row(w: Workload, b: int, t: int) -> np.ndarray:
    """Unrounded fp32 target logits of sequence b, position t (t = gamma_b is the bonus row)."""
    rng = _rng(w.wid, _T_TARGET, b, t)
    if w.recipe == "normal3":
        return rng.standard_normal(w.V, dtype=np.float32) * np.float32(3.0)
    if w.recipe == "normal4_mix":
        return rng.standard_normal(w.V, dtype=np.float32) * np.float32(4.0)
    if w.recipe == "normal5_resample":
        return rng.standard_normal(w.V, dtype=np.float32) * np.float32(5.0)
    if w.recipe == "zipf1.1":
        return _zipf_row(rng, w.V, 1.1)
    if w.recipe == "zipf1.2":
        return _zipf_row(rng, w.V, 1.2)
    raise ValueError(w.recipe)


def draft_row(w: Workload, b: int, t: int, tgt: np.ndarray) -> np.ndarray:
    """Unrounded fp32 draft logits derived from the unrounded target row of the same (b, t)."""
    rng = _rng(w.wid, _T_DRAFT, b, t)
    n = rng.standard_normal(w.V, dtype=np.float32)
    if w.recipe == "normal3":
        return tgt + n
    if w.recipe == "normal4_mix":
        return np.float32(0.8) * tgt + np.float32(1.5) * n
    if w.recipe == "zipf1.1":
        return tgt + n
    if w.recipe == "zipf1.2":
        return tgt + np.float32(1.2) * n
    if w.recipe == "normal5_resample":
        swap = rng.random(w.V, dtype=np.float32) < np.float32(0.1)
        return np.where(swap, n * np.float32(5.0), tgt)
    raise ValueError(w.recipe)


def _store(w: Workload, a: np.ndarray) -> np.ndarray:
    return a if w.dtype == "f32" else to_bf16_bits(a)


def np_dtype(w: Workload):
    return np.float32 if w.dtype == "f32" else np.uint16


@dataclass
class Round:
    workload: Workload
    rnd: int
    seqs: np.ndarray           # global sequence ids present, in order
    seq_off: np.ndarray        # int32 [B'+1]
    draft_logits: np.ndarray   # [N, V] float32 or uint16(bf16)
    tgt_logits: np.ndarray     # [N+B', V]
    uniforms: np.ndarray       # float32 [N+B']
    draft_uniforms: np.ndarray  # float32 [N]

    @property
    def B(self) -> int:
        return self.seq_off.shape[0] - 1

    @property
    def N(self) -> int:
        return int(self.seq_off[-1])


def build_round(w: Workload, rnd: int = 0, seqs=None, workers: int | None = None) -> Round:
    """Packed inputs of one round, for all sequences or for the listed global sequence ids."""
    g_all = gammas(w, rnd)
    seqs = np.arange(w.B, dtype=np.int64) if seqs is None else np.asarray(list(seqs), np.int64)
    g = g_all[seqs]
    off = seq_offsets(g)
    Bp, N = len(seqs), int(off[-1])
    draft = np.empty((N, w.V), np_dtype(w))
    tgt = np.empty((N + Bp, w.V), np_dtype(w))
    uni = np.empty(N + Bp, np.float32)
    duni = np.empty(N, np.float32)

    def fill(j: int) -> None:
        b = int(seqs[j])
        gb, d0 = int(g[j]), int(off[j])
        t0 = d0 + j
        uni[t0:t0 + gb + 1] = _rng(w.wid, _T_UNIFORM, rnd, b).random(w.gamma_max + 1, dtype=np.float32)[:gb + 1]
        duni[d0:d0 + gb] = _rng(w.wid, _T_DRAFT_UNIFORM, rnd, b).random(w.gamma_max, dtype=np.float32)[:gb]
        for t in range(gb + 1):
            tr = target_row(w, b, t)
            tgt[t0 + t] = _store(w, tr)
            if t < gb:
                draft[d0 + t] = _store(w, draft_row(w, b, t, tr))

    workers = workers or min(16, os.cpu_count() or 1)
    if Bp <= 1 or workers <= 1:
        for j in range(Bp):
            fill(j)
    else:
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(fill, range(Bp)))
    return Round(w, rnd, seqs, off, draft, tgt, uni, duni)
