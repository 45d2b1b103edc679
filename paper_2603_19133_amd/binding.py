"""ctypes binding of libpicospec.so with the same names as the C ABI (include/picospec.h).

Argument marshalling only: torch supplies device memory and the current stream, every step of
the path runs in the library's HIP kernels.  There is no fallback: if the library has not been
built (``python -m paper_2603_19133_amd.build``) importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpicospec.so")

F32, BF16 = 0, 1
OK, EINVAL, EWORKSPACE, EDTYPE, EHIP, EUNSUPPORTED, ESCRATCH = 0, -1, -2, -3, -4, -5, -6
FLAG_TOKEN_NOT_IN_SUPPORT, FLAG_NONFINITE, FLAG_RESIDUAL_EMPTY, FLAG_BAD_INPUT = 1, 2, 4, 8
CALL_COMPRESS, CALL_SAMPLE_DRAFT, CALL_VERIFY, CALL_SAMPLE_RESIDUAL = 0, 1, 2, 3
CALL_ROUND, CALL_VERIFY_SAMPLE = 6, 7
LIMIT_MAX_K, LIMIT_MAX_V = 0, 1
WIRE_FP32, WIRE_FP16, WIRE_BF16 = 0, 1, 2
WIRE_BAD_HEADER, WIRE_BAD_BATCH, WIRE_CLAMPED, WIRE_TRUNCATED = 1, 2, 4, 8

EXPORTS = ("picospec_round", "picospec_verify_sample", "picospec_verify_sample_static", "picospec_static_scratch_bytes", "picospec_compress", "picospec_sample_draft", "picospec_verify", "picospec_verify_range", "picospec_sample_residual",
           "picospec_row_stats", "picospec_compress_rejected", "picospec_resample_sparse",
           "picospec_pack_downlink", "picospec_unpack_downlink", "picospec_pack_uplink", "picospec_unpack_uplink",
           "picospec_downlink_bytes_max", "picospec_uplink_bytes", "picospec_max_load_byte", "picospec_check_device", "picospec_probe_clock",
           "picospec_workspace_bytes", "picospec_limit", "picospec_strerror", "picospec_version")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_19133_amd.build` "
                      "(there is no CPU fallback)")

lib = C.CDLL(LIB_PATH)

_p, _i32, _i64, _f, _sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
lib.picospec_compress.argtypes = [_p, C.c_int, _i64, _i32, _i32, _f, _i32, _f, _p, _p, _p, _p, _p, _p, _sz, _p]
lib.picospec_sample_draft.argtypes = [_p, _p, _p, _p, _i32, _i32, _p, _p, _p, _p]
lib.picospec_verify.argtypes = [_p, C.c_int, _i64, _i32, _f, _i32, _i32, _p, _p, _p, _p, _p, _p, _i32, C.c_int,
                                _p, _p, _p, _p, _p, _p, _p, _p, _p, _p, _sz, _p]
lib.picospec_verify_range.argtypes = [_p, C.c_int, _i64, _i32, _f, _i32, _i32, _p, _p, _p, _p, _p, _p, _i32, C.c_int,
                                      _p, _p, _p, _p, _i32, _p, _p, _p, _p, _p, _p, _p, _p, _sz, _p]
lib.picospec_round.argtypes = [_p, _p, C.c_int, _i64, _i64, _i32, _f, _i32, _i32, _p, _p, _i32, _f, C.c_int, _p,
                               _p, _p, _p, _p, _p, _p, _p, _p, _p, _p, _p, _p, _p, _p, _p, _p, _sz, _p]
lib.picospec_verify_sample.argtypes = [_p, C.c_int, _i64, _i32, _f, _i32, _i32, _p, _p, _p, _p, _p, _p, _i32, C.c_int, _p,
                                       _p, _p, _p, _p, _p, _p, _p, _p, _p, _p, _p, _sz, _p]
lib.picospec_verify_sample.restype = C.c_int
lib.picospec_verify_sample_static.argtypes = lib.picospec_verify_sample.argtypes[:-3] + [_p]
lib.picospec_verify_sample_static.restype = C.c_int
lib.picospec_static_scratch_bytes.argtypes = []
lib.picospec_static_scratch_bytes.restype = _i64
lib.picospec_sample_residual.argtypes = [_p, C.c_int, _i64, _i32, _f, _i32, _i32, _p, _p, _p, _p, _p, _p, _p, _p,
                                         _i32, C.c_int, _p, _p, _p, _p, _p, _sz, _p]
lib.picospec_row_stats.argtypes = [_p, C.c_int, _i64, _i32, _i32, _f, _p, _p, _p, _p]
lib.picospec_compress_rejected.argtypes = [_p, C.c_int, _i64, _i32, _f, _i32, _i32, _p, _p, _i32, _f,
                                           _p, _p, _p, _p, _p, _p, _sz, _p]
lib.picospec_resample_sparse.argtypes = [_p, C.c_int, _i64, _i32, _f, _i32, _i32, _p, _p, _p, _p, _p, _p, _p, _p,
                                         _i32, C.c_int, _p, _p, _p, _p, _p, _sz, _p]
lib.picospec_pack_downlink.argtypes = [_i32, _p, _p, _p, _p, _p, _p, _i32, C.c_int, _p, _i64, _p, _p, _p]
lib.picospec_unpack_downlink.argtypes = [_p, _i64, _i32, _i32, _p, _p, _p, _p, _p, _p, _p, _p]
lib.picospec_pack_uplink.argtypes = [_i32, _i32, _p, _p, _p, C.c_int, _p, _i64, _p, _p]
lib.picospec_unpack_uplink.argtypes = [_p, _i64, _i32, _i32, _p, _p, _p, _p, _p]
lib.picospec_downlink_bytes_max.argtypes = [_i32, _i32, C.c_int]
lib.picospec_downlink_bytes_max.restype = _i64
lib.picospec_uplink_bytes.argtypes = [_i32, _i32, C.c_int]
lib.picospec_uplink_bytes.restype = _i64
lib.picospec_max_load_byte.argtypes = [C.c_int, C.c_int, _i32, _i32]
lib.picospec_max_load_byte.restype = _i64
lib.picospec_check_device.argtypes = [_p, _sz, _p, _p]
lib.picospec_check_device.restype = C.c_int
lib.picospec_probe_clock.argtypes = [_p, _p]
lib.picospec_probe_clock.restype = C.c_int
lib.picospec_workspace_bytes.argtypes = [C.c_int, C.c_int, _i32, _i32, _i32]
lib.picospec_workspace_bytes.restype = _sz
lib.picospec_limit.argtypes = [C.c_int]
lib.picospec_limit.restype = _i64
lib.picospec_strerror.argtypes = [C.c_int]
lib.picospec_strerror.restype = C.c_char_p
for _n in ("picospec_compress", "picospec_sample_draft", "picospec_verify", "picospec_sample_residual",
           "picospec_row_stats", "picospec_compress_rejected", "picospec_resample_sparse", "picospec_version",
           "picospec_pack_downlink", "picospec_unpack_downlink", "picospec_pack_uplink", "picospec_unpack_uplink",
           "picospec_verify_range", "picospec_round"):
    getattr(lib, _n).restype = C.c_int


class PicoSpecError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"picospec error {code}: {lib.picospec_strerror(code).decode()}")


def _check(rc: int) -> None:
    if rc != OK:
        raise PicoSpecError(rc)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def alloc_workspace(dtype: torch.dtype, rows: int, V: int, device, which: int = CALL_VERIFY) -> torch.Tensor:
    """The optional workspace of verify / sample_residual / verify_sample / round for `rows` = n_draft + B target rows."""
    code = F32 if dtype == torch.float32 else BF16
    n = int(lib.picospec_workspace_bytes(which, code, rows, V, 0))
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device)


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise PicoSpecError(EDTYPE)


def _logits_2d(t: torch.Tensor):
    if t.dim() != 2 or not t.is_cuda:
        raise PicoSpecError(EINVAL)
    if t.shape[0] == 0:                       # no rows: the strides of an empty tensor mean nothing
        return _dtype_code(t), t.shape[1]
    if t.stride(1) != 1:
        raise PicoSpecError(EINVAL)
    return _dtype_code(t), t.stride(0)


@dataclass
class Compressed:
    idx: torch.Tensor     # int32 [rows, k]
    prob: torch.Tensor    # float32 [rows, k]
    count: torch.Tensor   # int32 [rows]
    mass: torch.Tensor    # float32 [rows]
    lse: torch.Tensor     # float32 [rows]
    k: int


def alloc_compressed(rows: int, k: int, device) -> Compressed:
    e = lambda *s, dt=torch.float32: torch.empty(*s, dtype=dt, device=device)
    return Compressed(e(rows, k, dt=torch.int32), e(rows, k), e(rows, dt=torch.int32), e(rows), e(rows), k)


def compress(logits: torch.Tensor, V: int, temperature: float, k: int, top_p: float = 0.0,
             out: Compressed | None = None) -> Compressed:
    """picospec_compress on [rows, >=V] fp32/bf16 device logits."""
    dt, ld = _logits_2d(logits)
    rows = logits.shape[0]
    out = out or alloc_compressed(rows, k, logits.device)
    _check(lib.picospec_compress(_ptr(logits), dt, ld, rows, V, temperature, k, top_p,
                                 _ptr(out.idx), _ptr(out.prob), _ptr(out.count), _ptr(out.mass), _ptr(out.lse),
                                 None, 0, _stream()))
    return out


def sample_draft(q: Compressed, uniforms: torch.Tensor, tok: torch.Tensor | None = None,
                 q_scalar: torch.Tensor | None = None):
    """picospec_sample_draft -> (tok int32 [rows], q_scalar float32 [rows])."""
    rows = q.idx.shape[0]
    tok = tok if tok is not None else torch.empty(rows, dtype=torch.int32, device=q.idx.device)
    q_scalar = q_scalar if q_scalar is not None else torch.empty(rows, dtype=torch.float32, device=q.idx.device)
    _check(lib.picospec_sample_draft(_ptr(q.idx), _ptr(q.prob), _ptr(q.count), _ptr(q.mass), q.k, rows,
                                     _ptr(uniforms), _ptr(tok), _ptr(q_scalar), _stream()))
    return tok, q_scalar


@dataclass
class Verified:
    n_accept: torch.Tensor   # int32 [B]
    p_tok: torch.Tensor      # float32 [N]
    q_tok: torch.Tensor      # float32 [N]
    tgt_max: torch.Tensor    # float32 [N+B]
    tgt_sum: torch.Tensor    # float32 [N+B]
    tgt_lse: torch.Tensor    # float32 [N+B]
    flags: torch.Tensor      # int32 (bit pattern of uint32) [B]


def alloc_verified(B: int, N: int, device) -> Verified:
    e = lambda n, dt=torch.float32: torch.empty(n, dtype=dt, device=device)
    return Verified(e(B, torch.int32), e(N), e(N), e(N + B), e(N + B), e(N + B), e(B, torch.int32))


def verify(tgt_logits: torch.Tensor, V: int, temperature: float, seq_off: torch.Tensor, n_draft: int,
           draft_tok: torch.Tensor, q: Compressed | None, uniforms: torch.Tensor, renorm: int = 1,
           q_scalar: torch.Tensor | None = None, out: Verified | None = None,
           workspace: torch.Tensor | None = None) -> Verified:
    """picospec_verify; seq_off int32 [B+1] on device, n_draft = seq_off[B] known on the host.  `workspace`
    (alloc_workspace) receives the target rows' segment table for sample_residual."""
    dt, ld = _logits_2d(tgt_logits)
    B = seq_off.shape[0] - 1
    out = out or alloc_verified(B, n_draft, tgt_logits.device)
    _check(lib.picospec_verify(_ptr(tgt_logits), dt, ld, V, temperature, B, n_draft, _ptr(seq_off), _ptr(draft_tok),
                               _ptr(q.idx) if q else None, _ptr(q.prob) if q else None,
                               _ptr(q.count) if q else None, _ptr(q.mass) if q else None,
                               q.k if q else 0, renorm, _ptr(q_scalar), _ptr(uniforms),
                               _ptr(out.n_accept), _ptr(out.p_tok), _ptr(out.q_tok),
                               _ptr(out.tgt_max), _ptr(out.tgt_sum), _ptr(out.tgt_lse), _ptr(out.flags),
                               _ptr(workspace), _nbytes(workspace), _stream()))
    return out


def verify_range(tgt_logits: torch.Tensor, V: int, temperature: float, seq_off: torch.Tensor, n_draft: int,
                 draft_tok: torch.Tensor, q: Compressed | None, uniforms: torch.Tensor,
                 pos_begin: torch.Tensor | None, pos_end: torch.Tensor | None, gamma_max: int, renorm: int = 1,
                 q_scalar: torch.Tensor | None = None, out: Verified | None = None) -> Verified:
    """picospec_verify_range: the draft positions pos_begin[b] <= t < pos_end[b] only; `out` from an earlier
    call keeps its entries outside the range."""
    dt, ld = _logits_2d(tgt_logits)
    B = seq_off.shape[0] - 1
    out = out or alloc_verified(B, n_draft, tgt_logits.device)
    _check(lib.picospec_verify_range(_ptr(tgt_logits), dt, ld, V, temperature, B, n_draft, _ptr(seq_off), _ptr(draft_tok),
                                     _ptr(q.idx) if q else None, _ptr(q.prob) if q else None,
                                     _ptr(q.count) if q else None, _ptr(q.mass) if q else None,
                                     q.k if q else 0, renorm, _ptr(q_scalar), _ptr(uniforms),
                                     _ptr(pos_begin), _ptr(pos_end), gamma_max,
                                     _ptr(out.n_accept), _ptr(out.p_tok), _ptr(out.q_tok),
                                     _ptr(out.tgt_max), _ptr(out.tgt_sum), _ptr(out.tgt_lse), _ptr(out.flags),
                                     None, 0, _stream()))
    return out


def round(draft_logits: torch.Tensor, tgt_logits: torch.Tensor, V: int, temperature: float, seq_off: torch.Tensor,
          n_draft: int, draft_tok: torch.Tensor, k: int, uniforms: torch.Tensor, top_p: float = 0.0, renorm: int = 1,
          q: "Compressed | None" = None, ver: "Verified | None" = None, res: "Residual | None" = None,
          workspace: torch.Tensor | None = None):
    """picospec_round -> (Compressed, Verified, Residual): the whole round in one call."""
    dt, ld_d = _logits_2d(draft_logits) if n_draft else (_dtype_code(tgt_logits), V)
    dt_t, ld_t = _logits_2d(tgt_logits)
    if dt != dt_t:
        raise PicoSpecError(EDTYPE)
    B = seq_off.shape[0] - 1
    dev = tgt_logits.device
    q = q or alloc_compressed(n_draft, k, dev)
    ver = ver or alloc_verified(B, n_draft, dev)
    res = res or alloc_residual(B, dev)
    _check(lib.picospec_round(_ptr(draft_logits), _ptr(tgt_logits), dt, ld_d, ld_t, V, temperature, B, n_draft,
                              _ptr(seq_off), _ptr(draft_tok), k, top_p, renorm, _ptr(uniforms),
                              _ptr(q.idx), _ptr(q.prob), _ptr(q.count), _ptr(q.mass), _ptr(q.lse),
                              _ptr(ver.n_accept), _ptr(ver.p_tok), _ptr(ver.q_tok),
                              _ptr(ver.tgt_max), _ptr(ver.tgt_sum), _ptr(ver.tgt_lse), _ptr(ver.flags),
                              _ptr(res.out_tok), _ptr(res.resid_mass), _ptr(res.flags),
                              _ptr(workspace), _nbytes(workspace), _stream()))
    return q, ver, res


def verify_sample(tgt_logits: torch.Tensor, V: int, temperature: float, seq_off: torch.Tensor, n_draft: int,
                  draft_tok: torch.Tensor, q: "Compressed", uniforms: torch.Tensor, renorm: int = 1,
                  ver: "Verified | None" = None, res: "Residual | None" = None, workspace: torch.Tensor | None = None):
    """picospec_verify_sample -> (Verified, Residual): verification and draw on records that exist."""
    dt, ld = _logits_2d(tgt_logits)
    B = seq_off.shape[0] - 1
    dev = tgt_logits.device
    ver = ver or alloc_verified(B, n_draft, dev)
    res = res or alloc_residual(B, dev)
    _check(lib.picospec_verify_sample(_ptr(tgt_logits), dt, ld, V, temperature, B, n_draft, _ptr(seq_off), _ptr(draft_tok),
                                      _ptr(q.idx), _ptr(q.prob), _ptr(q.count), _ptr(q.mass), q.k, renorm, _ptr(uniforms),
                                      _ptr(ver.n_accept), _ptr(ver.p_tok), _ptr(ver.q_tok),
                                      _ptr(ver.tgt_max), _ptr(ver.tgt_sum), _ptr(ver.tgt_lse), _ptr(ver.flags),
                                      _ptr(res.out_tok), _ptr(res.resid_mass), _ptr(res.flags),
                                      _ptr(workspace), _nbytes(workspace), _stream()))
    return ver, res


@dataclass
class Residual:
    out_tok: torch.Tensor     # int32 [B]
    resid_mass: torch.Tensor  # float32 [B]
    flags: torch.Tensor       # int32 [B]


def alloc_residual(B: int, device) -> Residual:
    return Residual(torch.empty(B, dtype=torch.int32, device=device),
                    torch.empty(B, dtype=torch.float32, device=device),
                    torch.empty(B, dtype=torch.int32, device=device))


def verify_sample_static(tgt_logits: torch.Tensor, V: int, temperature: float, seq_off: torch.Tensor, n_draft: int,
                         draft_tok: torch.Tensor, q: "Compressed", uniforms: torch.Tensor, ver: "Verified", res: "Residual",
                         renorm: int = 1) -> None:
    """picospec_verify_sample_static into `ver` and `res` (the caller's: this wrapper allocates nothing either)."""
    dt, ld = _logits_2d(tgt_logits)
    B = seq_off.shape[0] - 1
    _check(lib.picospec_verify_sample_static(_ptr(tgt_logits), dt, ld, V, temperature, B, n_draft, _ptr(seq_off), _ptr(draft_tok),
                                             _ptr(q.idx), _ptr(q.prob), _ptr(q.count), _ptr(q.mass), q.k, renorm, _ptr(uniforms),
                                             _ptr(ver.n_accept), _ptr(ver.p_tok), _ptr(ver.q_tok),
                                             _ptr(ver.tgt_max), _ptr(ver.tgt_sum), _ptr(ver.tgt_lse), _ptr(ver.flags),
                                             _ptr(res.out_tok), _ptr(res.resid_mass), _ptr(res.flags), _stream()))


def static_scratch_bytes() -> int:
    return int(lib.picospec_static_scratch_bytes())


def sample_residual(tgt_logits: torch.Tensor, V: int, temperature: float, seq_off: torch.Tensor, n_draft: int,
                    ver: Verified, q: Compressed, uniforms: torch.Tensor, renorm: int = 1,
                    out: Residual | None = None, n_accept: torch.Tensor | None = None,
                    workspace: torch.Tensor | None = None) -> Residual:
    """picospec_sample_residual from the statistics and first-rejection indices of `ver` (and, if given, from the
    segment table that verify left in `workspace`)."""
    dt, ld = _logits_2d(tgt_logits)
    B = seq_off.shape[0] - 1
    out = out or alloc_residual(B, tgt_logits.device)
    na = ver.n_accept if n_accept is None else n_accept
    _check(lib.picospec_sample_residual(_ptr(tgt_logits), dt, ld, V, temperature, B, n_draft, _ptr(seq_off), _ptr(na),
                                        _ptr(ver.tgt_max), _ptr(ver.tgt_sum),
                                        _ptr(q.idx), _ptr(q.prob), _ptr(q.count), _ptr(q.mass), q.k, renorm,
                                        _ptr(uniforms), _ptr(out.out_tok), _ptr(out.resid_mass), _ptr(out.flags),
                                        _ptr(workspace), _nbytes(workspace), _stream()))
    return out


def row_stats(logits: torch.Tensor, V: int, temperature: float):
    """picospec_row_stats -> (row_max, row_sum, row_lse), float32 [rows] each."""
    dt, ld = _logits_2d(logits)
    rows = logits.shape[0]
    e = lambda: torch.empty(rows, dtype=torch.float32, device=logits.device)
    mx, sm, ls = e(), e(), e()
    _check(lib.picospec_row_stats(_ptr(logits), dt, ld, rows, V, temperature, _ptr(mx), _ptr(sm), _ptr(ls), _stream()))
    return mx, sm, ls


def compress_rejected(tgt_logits: torch.Tensor, V: int, temperature: float, seq_off: torch.Tensor, n_draft: int,
                      n_accept: torch.Tensor, k: int, top_p: float = 0.0, out: Compressed | None = None) -> Compressed:
    """picospec_compress_rejected: the downlink record of every sequence's rejected (or bonus) target row."""
    dt, ld = _logits_2d(tgt_logits)
    B = seq_off.shape[0] - 1
    out = out or alloc_compressed(B, k, tgt_logits.device)
    _check(lib.picospec_compress_rejected(_ptr(tgt_logits), dt, ld, V, temperature, B, n_draft, _ptr(seq_off),
                                          _ptr(n_accept), k, top_p, _ptr(out.idx), _ptr(out.prob), _ptr(out.count),
                                          _ptr(out.mass), _ptr(out.lse), None, 0, _stream()))
    return out


def resample_sparse(draft_logits: torch.Tensor, V: int, temperature: float, seq_off: torch.Tensor, n_draft: int,
                    n_accept: torch.Tensor, draft_max: torch.Tensor, draft_sum: torch.Tensor, p: Compressed,
                    uniforms: torch.Tensor, renorm: int = 0, out: Residual | None = None) -> Residual:
    """picospec_resample_sparse: the edge's local draw from norm(max(0, P_j - Q_j)) on the record's slots."""
    dt, ld = _logits_2d(draft_logits)
    B = seq_off.shape[0] - 1
    out = out or alloc_residual(B, draft_logits.device)
    _check(lib.picospec_resample_sparse(_ptr(draft_logits), dt, ld, V, temperature, B, n_draft, _ptr(seq_off),
                                        _ptr(n_accept), _ptr(draft_max), _ptr(draft_sum),
                                        _ptr(p.idx), _ptr(p.prob), _ptr(p.count), _ptr(p.mass), p.k, renorm,
                                        _ptr(uniforms), _ptr(out.out_tok), _ptr(out.resid_mass), _ptr(out.flags),
                                        None, 0, _stream()))
    return out


def downlink_bytes_max(B: int, k: int, prob_format: int) -> int:
    return lib.picospec_downlink_bytes_max(B, k, prob_format)


def uplink_bytes(B: int, n_draft: int, prob_format: int) -> int:
    return lib.picospec_uplink_bytes(B, n_draft, prob_format)


def pack_downlink(seq_off: torch.Tensor, n_accept: torch.Tensor, token: torch.Tensor | None,
                  rec: Compressed | None, prob_format: int, wire: torch.Tensor | None = None):
    """picospec_pack_downlink -> (wire uint8 [capacity], wire_bytes int64 [1], status int32 [1]), all on device."""
    B = seq_off.shape[0] - 1
    k = rec.k if rec is not None else 0
    dev = seq_off.device
    if wire is None:
        wire = torch.empty(downlink_bytes_max(B, k, prob_format), dtype=torch.uint8, device=dev)
    nbytes = torch.empty(1, dtype=torch.int64, device=dev)
    status = torch.empty(1, dtype=torch.int32, device=dev)
    _check(lib.picospec_pack_downlink(B, _ptr(seq_off), _ptr(n_accept), _ptr(token),
                                      _ptr(rec.idx) if rec else None, _ptr(rec.prob) if rec else None,
                                      _ptr(rec.count) if rec else None, k, prob_format,
                                      _ptr(wire), wire.numel(), _ptr(nbytes), _ptr(status), _stream()))
    return wire, nbytes, status


@dataclass
class Downlink:
    n_accept: torch.Tensor   # int32 [B]
    token: torch.Tensor      # int32 [B]
    rec: Compressed          # idx/prob [B,k], count, mass (lse unused)
    status: torch.Tensor     # int32 [1]


def unpack_downlink(wire: torch.Tensor, wire_bytes: int, B: int, k: int) -> Downlink:
    """picospec_unpack_downlink; `wire_bytes` is the received length (a host value)."""
    dev = wire.device
    out = Downlink(torch.empty(B, dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
                   alloc_compressed(B, k, dev), torch.empty(1, dtype=torch.int32, device=dev))
    _check(lib.picospec_unpack_downlink(_ptr(wire), wire_bytes, B, k, _ptr(out.n_accept), _ptr(out.token),
                                        _ptr(out.rec.idx), _ptr(out.rec.prob), _ptr(out.rec.count),
                                        _ptr(out.rec.mass), _ptr(out.status), _stream()))
    return out


def pack_uplink(seq_off: torch.Tensor, n_draft: int, draft_tok: torch.Tensor, q_scalar: torch.Tensor,
                prob_format: int, wire: torch.Tensor | None = None):
    """picospec_pack_uplink -> (wire uint8, wire_bytes int64 [1]) on device."""
    B = seq_off.shape[0] - 1
    dev = seq_off.device
    if wire is None:
        wire = torch.empty(uplink_bytes(B, n_draft, prob_format), dtype=torch.uint8, device=dev)
    nbytes = torch.empty(1, dtype=torch.int64, device=dev)
    _check(lib.picospec_pack_uplink(B, n_draft, _ptr(seq_off), _ptr(draft_tok), _ptr(q_scalar), prob_format,
                                    _ptr(wire), wire.numel(), _ptr(nbytes), _stream()))
    return wire, nbytes


def unpack_uplink(wire: torch.Tensor, wire_bytes: int, B: int, n_max: int):
    """picospec_unpack_uplink -> (seq_off int32 [B+1], draft_tok int32 [n_max], q_scalar float32 [n_max], status)."""
    dev = wire.device
    seq_off = torch.empty(B + 1, dtype=torch.int32, device=dev)
    tok = torch.empty(n_max, dtype=torch.int32, device=dev)
    q = torch.empty(n_max, dtype=torch.float32, device=dev)
    status = torch.empty(1, dtype=torch.int32, device=dev)
    _check(lib.picospec_unpack_uplink(_ptr(wire), wire_bytes, B, n_max, _ptr(seq_off), _ptr(tok), _ptr(q),
                                      _ptr(status), _stream()))
    return seq_off, tok, q, status


def check_device(device) -> int:
    """picospec_check_device -> status word (0: the device's buffer loads range-check as the row kernels assume)."""
    ws = torch.empty(64 * 1024, dtype=torch.uint8, device=device)
    status = torch.full((1,), -1, dtype=torch.int32, device=device)
    _check(lib.picospec_check_device(_ptr(ws), ws.numel(), _ptr(status), _stream()))
    return int(status.item()) & 0xFFFFFFFF


def probe_clock(ticks: torch.Tensor) -> None:
    """picospec_probe_clock into `ticks` (int64 [2], device): 100 * ticks[0] / ticks[1] = shader clock in MHz."""
    _check(lib.picospec_probe_clock(_ptr(ticks), _stream()))


def max_load_byte(which: int, dtype: int, V: int, misalign_bytes: int) -> int:
    return int(lib.picospec_max_load_byte(which, dtype, V, misalign_bytes))


def workspace_bytes(which: int, dtype: int, rows: int, V: int, k: int) -> int:
    return int(lib.picospec_workspace_bytes(which, dtype, rows, V, k))


def limit(which: int) -> int:
    return int(lib.picospec_limit(which))


def version() -> int:
    return int(lib.picospec_version())
