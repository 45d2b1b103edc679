"""CPU oracle for the PicoSpec separate-rejection-sampling path.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py``.  Nothing in the product package imports this, and this module
(the oracle proper) imports nothing from the product package.  ``oracle/downlink_bias.py``, a script that tabulates
the truncation bias of a K-entry record on synthetic rounds with the oracle alone, takes its inputs from the seeded
input generators (``paper_2603_19133_amd/workloads.py``, which hold none of the method's arithmetic).

The arithmetic lives in ``picospec_oracle.c`` (plain C, fp64) and the wire formats in
``picospec_wire_oracle.c``; this module only builds them with gcc and marshals numpy arrays into them.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "picospec_oracle.c")
_SRC_WIRE = os.path.join(_HERE, "picospec_wire_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

F32, BF16 = 0, 1
FLAG_TOKEN_NOT_IN_SUPPORT, FLAG_NONFINITE, FLAG_RESIDUAL_EMPTY = 1, 2, 4


def build() -> str:
    """Compile the C oracle (no fast-math, so libm exp/log and IEEE ordering are kept)."""
    cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
           "-o", _LIB, _SRC, _SRC_WIRE, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_WIRE)):
            build()
        _lib = C.CDLL(_LIB)
        for name in ("oracle_compress", "oracle_sample_draft", "oracle_verify",
                     "oracle_sample_residual", "oracle_resample_sparse", "oracle_record_bytes",
                     "oracle_wire_quantise", "oracle_pack_downlink", "oracle_unpack_downlink",
                     "oracle_pack_uplink", "oracle_unpack_uplink"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def threads() -> int:
    """Host threads the OpenMP loops use (what ``cores`` in the bench line reports)."""
    n = os.environ.get("OMP_NUM_THREADS")
    return int(n) if n else (os.cpu_count() or 1)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _logits(a: np.ndarray):
    """Accepts float32 [rows, ld] or uint16 [rows, ld] holding bf16 bit patterns."""
    assert a.ndim == 2 and a.flags.c_contiguous
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"logits must be float32 or uint16(bf16 bits), got {a.dtype}")


@dataclass
class Compressed:
    idx: np.ndarray      # int32 [rows, k]
    prob: np.ndarray     # float64 [rows, k]
    count: np.ndarray    # int32 [rows]
    mass: np.ndarray     # float64 [rows]
    lse: np.ndarray      # float64 [rows]
    topp_margin: np.ndarray  # float64 [rows]
    k: int


def compress(logits: np.ndarray, V: int, T: float, k: int, top_p: float = 0.0) -> Compressed:
    dt = _logits(logits)
    n, ld = logits.shape
    out = Compressed(np.empty((n, k), np.int32), np.empty((n, k), np.float64),
                     np.empty(n, np.int32), np.empty(n, np.float64), np.empty(n, np.float64),
                     np.empty(n, np.float64), k)
    rc = lib().oracle_compress(_ptr(logits), C.c_int(dt), C.c_int64(ld), C.c_int32(n), C.c_int32(V),
                               C.c_double(T), C.c_int32(k), C.c_double(top_p),
                               _ptr(out.idx), _ptr(out.prob), _ptr(out.count), _ptr(out.mass),
                               _ptr(out.lse), _ptr(out.topp_margin))
    if rc != 0:
        raise ValueError(f"oracle_compress rc={rc}")
    return out


def sample_draft(q: Compressed, uniforms: np.ndarray):
    """-> (tok int32 [rows], slot int32 [rows], cdf_margin float64 [rows])."""
    n = q.idx.shape[0]
    u = np.ascontiguousarray(uniforms, np.float32)
    assert u.shape == (n,)
    tok, slot, mar = np.empty(n, np.int32), np.empty(n, np.int32), np.empty(n, np.float64)
    rc = lib().oracle_sample_draft(_ptr(q.idx), _ptr(q.prob), _ptr(q.count), C.c_int32(q.k),
                                   C.c_int32(n), _ptr(u), _ptr(tok), _ptr(slot), _ptr(mar))
    if rc != 0:
        raise ValueError(f"oracle_sample_draft rc={rc}")
    return tok, slot, mar


@dataclass
class Verified:
    n_accept: np.ndarray   # int32 [B]
    p_tok: np.ndarray      # float64 [N]
    q_tok: np.ndarray      # float64 [N]
    tgt_lse: np.ndarray    # float64 [N+B]
    flags: np.ndarray      # uint32 [B]
    margin: np.ndarray     # float64 [N]


def verify(tgt_logits: np.ndarray, V: int, T: float, seq_off: np.ndarray, draft_tok: np.ndarray,
           q: Compressed | None, uniforms: np.ndarray, renorm: int = 1,
           q_scalar: np.ndarray | None = None, pos_begin: np.ndarray | None = None,
           pos_end: np.ndarray | None = None, out: Verified | None = None) -> Verified:
    """pos_begin / pos_end restrict every sequence to a range of its draft positions; `out` (the result of an
    earlier call) is then updated in place, entries outside the range keep their values."""
    dt = _logits(tgt_logits)
    rows, ld = tgt_logits.shape
    seq_off = np.ascontiguousarray(seq_off, np.int32)
    B = seq_off.shape[0] - 1
    N = int(seq_off[-1])
    assert rows >= N + B
    draft_tok = np.ascontiguousarray(draft_tok, np.int32)
    u = np.ascontiguousarray(uniforms, np.float32)
    assert draft_tok.shape == (N,) and u.shape[0] >= N + B
    qs = None if q_scalar is None else np.ascontiguousarray(q_scalar, np.float64)
    if out is None:
        out = Verified(np.full(B, -7, np.int32), np.full(N, np.nan), np.full(N, np.nan),
                       np.full(N + B, np.nan), np.zeros(B, np.uint32), np.full(N, np.nan))
    pb = None if pos_begin is None else np.ascontiguousarray(pos_begin, np.int32)
    pe = None if pos_end is None else np.ascontiguousarray(pos_end, np.int32)
    k = q.k if q is not None else 1
    rc = lib().oracle_verify(_ptr(tgt_logits), C.c_int(dt), C.c_int64(ld), C.c_int32(V), C.c_double(T),
                             C.c_int32(B), _ptr(seq_off), _ptr(draft_tok),
                             _ptr(q.idx) if q else None, _ptr(q.prob) if q else None,
                             _ptr(q.count) if q else None, _ptr(q.mass) if q else None,
                             C.c_int32(k), C.c_int(renorm), _ptr(qs), _ptr(u),
                             _ptr(out.n_accept), _ptr(out.p_tok), _ptr(out.q_tok), _ptr(out.tgt_lse),
                             _ptr(out.flags), _ptr(out.margin), _ptr(pb), _ptr(pe))
    if rc != 0:
        raise ValueError(f"oracle_verify rc={rc}")
    return out


@dataclass
class Residual:
    out_tok: np.ndarray     # int32 [B]
    resid_mass: np.ndarray  # float64 [B]
    flags: np.ndarray       # uint32 [B]
    cdf_margin: np.ndarray  # float64 [B]


def sample_residual(tgt_logits: np.ndarray, V: int, T: float, seq_off: np.ndarray,
                    n_accept: np.ndarray, tgt_lse: np.ndarray, q: Compressed,
                    uniforms: np.ndarray, renorm: int = 1) -> Residual:
    dt = _logits(tgt_logits)
    _, ld = tgt_logits.shape
    seq_off = np.ascontiguousarray(seq_off, np.int32)
    B = seq_off.shape[0] - 1
    n_accept = np.ascontiguousarray(n_accept, np.int32)
    tgt_lse = np.ascontiguousarray(tgt_lse, np.float64)
    u = np.ascontiguousarray(uniforms, np.float32)
    out = Residual(np.empty(B, np.int32), np.empty(B, np.float64), np.zeros(B, np.uint32),
                   np.empty(B, np.float64))
    rc = lib().oracle_sample_residual(_ptr(tgt_logits), C.c_int(dt), C.c_int64(ld), C.c_int32(V),
                                      C.c_double(T), C.c_int32(B), _ptr(seq_off), _ptr(n_accept),
                                      _ptr(tgt_lse), _ptr(q.idx), _ptr(q.prob), _ptr(q.count),
                                      _ptr(q.mass), C.c_int32(q.k), C.c_int(renorm), _ptr(u),
                                      _ptr(out.out_tok), _ptr(out.resid_mass), _ptr(out.flags),
                                      _ptr(out.cdf_margin))
    if rc != 0:
        raise ValueError(f"oracle_sample_residual rc={rc}")
    return out


def rejected_rows(seq_off: np.ndarray, n_accept: np.ndarray) -> np.ndarray:
    """Target row of sequence b at its first rejected (or bonus) position: seq_off[b] + b + n_accept[b]."""
    seq_off = np.asarray(seq_off, np.int64)
    B = seq_off.shape[0] - 1
    return seq_off[:B] + np.arange(B, dtype=np.int64) + np.asarray(n_accept, np.int64)


def compress_rejected(tgt_logits: np.ndarray, V: int, T: float, seq_off: np.ndarray, n_accept: np.ndarray,
                      k: int, top_p: float = 0.0) -> Compressed:
    """The downlink record (Eq. 4): Top-K of the target distribution at each sequence's rejected position."""
    rows = rejected_rows(seq_off, n_accept)
    return compress(np.ascontiguousarray(tgt_logits[rows]), V, T, k, top_p)


@dataclass
class SparseResample:
    out_tok: np.ndarray     # int32 [B]
    resid_mass: np.ndarray  # float64 [B]
    flags: np.ndarray       # uint32 [B]
    cdf_margin: np.ndarray  # float64 [B]
    weights: np.ndarray     # float64 [B,k]: the per-slot weights drawn from


def resample_sparse(draft_logits: np.ndarray, V: int, T: float, seq_off: np.ndarray, n_accept: np.ndarray,
                    p: Compressed, uniforms: np.ndarray, renorm: int = 0) -> SparseResample:
    dt = _logits(draft_logits)
    _, ld = draft_logits.shape
    seq_off = np.ascontiguousarray(seq_off, np.int32)
    B = seq_off.shape[0] - 1
    n_accept = np.ascontiguousarray(n_accept, np.int32)
    u = np.ascontiguousarray(uniforms, np.float32)
    out = SparseResample(np.empty(B, np.int32), np.empty(B, np.float64), np.zeros(B, np.uint32),
                         np.empty(B, np.float64), np.zeros((B, p.k), np.float64))
    rc = lib().oracle_resample_sparse(_ptr(draft_logits), C.c_int(dt), C.c_int64(ld), C.c_int32(V),
                                      C.c_double(T), C.c_int32(B), _ptr(seq_off), _ptr(n_accept),
                                      _ptr(p.idx), _ptr(p.prob), _ptr(p.count), _ptr(p.mass),
                                      C.c_int32(p.k), C.c_int(renorm), _ptr(u),
                                      _ptr(out.out_tok), _ptr(out.resid_mass), _ptr(out.flags),
                                      _ptr(out.cdf_margin), _ptr(out.weights))
    if rc != 0:
        raise ValueError(f"oracle_resample_sparse rc={rc}")
    return out


def record_bytes() -> int:
    return lib().oracle_record_bytes()


# ---- wire messages (picospec_wire_oracle.c)

WIRE_FP32, WIRE_FP16, WIRE_BF16 = 0, 1, 2
WIRE_BAD_HEADER, WIRE_BAD_BATCH, WIRE_CLAMPED, WIRE_TRUNCATED = 1, 2, 4, 8


def wire_quantise(values: np.ndarray, fmt: int):
    """fp32 -> (bits uint16, value read back float64) in the wire's fp16 or bf16."""
    v = np.ascontiguousarray(values, np.float32).ravel()
    bits, back = np.empty(v.size, np.uint16), np.empty(v.size, np.float64)
    rc = lib().oracle_wire_quantise(_ptr(v), C.c_int32(v.size), C.c_int(fmt), _ptr(bits), _ptr(back))
    if rc != 0:
        raise ValueError(f"oracle_wire_quantise rc={rc}")
    return bits, back


def pack_downlink(seq_off: np.ndarray, n_accept: np.ndarray, token: np.ndarray | None,
                  idx: np.ndarray | None, prob: np.ndarray | None, count: np.ndarray | None,
                  fmt: int, capacity: int | None = None):
    """-> (message bytes uint8 [wire_bytes], wire_bytes); the record arrays are [B,k] int32 / float32."""
    seq_off = np.ascontiguousarray(seq_off, np.int32)
    B = seq_off.shape[0] - 1
    n_accept = np.ascontiguousarray(n_accept, np.int32)
    token = None if token is None else np.ascontiguousarray(token, np.int32)
    k = 0
    if idx is not None:
        idx = np.ascontiguousarray(idx, np.int32)
        prob = np.ascontiguousarray(prob, np.float32)
        count = np.ascontiguousarray(count, np.int32)
        k = idx.shape[1]
        assert idx.shape == (B, k) and prob.shape == (B, k) and count.shape == (B,)
    cap = 8 + 8 * B + 8 * B * k + 4 if capacity is None else capacity
    wire = np.full(max(cap, 1), 0xEE, np.uint8)
    nbytes = C.c_int64(0)
    rc = lib().oracle_pack_downlink(C.c_int32(B), _ptr(seq_off), _ptr(n_accept), _ptr(token), _ptr(idx), _ptr(prob),
                                    _ptr(count), C.c_int32(k), C.c_int(fmt), _ptr(wire), C.c_int64(cap),
                                    C.byref(nbytes))
    if rc < 0:
        raise ValueError(f"oracle_pack_downlink rc={rc}")
    return (wire[:nbytes.value].copy() if rc == 0 else None), nbytes.value


@dataclass
class Downlink:
    n_accept: np.ndarray   # int32 [B]
    token: np.ndarray      # int32 [B]
    idx: np.ndarray        # int32 [B,k]
    prob: np.ndarray       # float64 [B,k]
    count: np.ndarray      # int32 [B]
    mass: np.ndarray       # float64 [B]
    status: int


def unpack_downlink(wire: np.ndarray, B: int, k: int) -> Downlink:
    wire = np.ascontiguousarray(wire, np.uint8)
    out = Downlink(np.full(B, -7, np.int32), np.full(B, -7, np.int32), np.full((B, k), -7, np.int32),
                   np.full((B, k), -7.0, np.float64), np.full(B, -7, np.int32), np.full(B, -7.0, np.float64), 0)
    st = C.c_uint32(0)
    rc = lib().oracle_unpack_downlink(_ptr(wire), C.c_int64(wire.size), C.c_int32(B), C.c_int32(k),
                                      _ptr(out.n_accept), _ptr(out.token), _ptr(out.idx), _ptr(out.prob),
                                      _ptr(out.count), _ptr(out.mass), C.byref(st))
    if rc != 0:
        raise ValueError(f"oracle_unpack_downlink rc={rc}")
    out.status = st.value
    return out


def pack_uplink(seq_off: np.ndarray, draft_tok: np.ndarray, q_scalar: np.ndarray, fmt: int,
                capacity: int | None = None):
    seq_off = np.ascontiguousarray(seq_off, np.int32)
    B = seq_off.shape[0] - 1
    draft_tok = np.ascontiguousarray(draft_tok, np.int32)
    q_scalar = np.ascontiguousarray(q_scalar, np.float32)
    N = int(seq_off[-1])
    cap = 8 + 2 * B + 4 + 8 * N + 4 if capacity is None else capacity
    wire = np.full(max(cap, 1), 0xEE, np.uint8)
    nbytes = C.c_int64(0)
    rc = lib().oracle_pack_uplink(C.c_int32(B), _ptr(seq_off), _ptr(draft_tok), _ptr(q_scalar), C.c_int(fmt),
                                  _ptr(wire), C.c_int64(cap), C.byref(nbytes))
    if rc < 0:
        raise ValueError(f"oracle_pack_uplink rc={rc}")
    return (wire[:nbytes.value].copy() if rc == 0 else None), nbytes.value


@dataclass
class Uplink:
    seq_off: np.ndarray    # int32 [B+1]
    draft_tok: np.ndarray  # int32 [n_max]
    q_scalar: np.ndarray   # float64 [n_max]
    status: int


def unpack_uplink(wire: np.ndarray, B: int, n_max: int) -> Uplink:
    wire = np.ascontiguousarray(wire, np.uint8)
    out = Uplink(np.full(B + 1, -7, np.int32), np.full(n_max, -7, np.int32), np.full(n_max, -7.0, np.float64), 0)
    st = C.c_uint32(0)
    rc = lib().oracle_unpack_uplink(_ptr(wire), C.c_int64(wire.size), C.c_int32(B), C.c_int32(n_max),
                                    _ptr(out.seq_off), _ptr(out.draft_tok), _ptr(out.q_scalar), C.byref(st))
    if rc != 0:
        raise ValueError(f"oracle_unpack_uplink rc={rc}")
    out.status = st.value
    return out
