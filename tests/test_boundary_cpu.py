"""The C-ABI library without a GPU: it loads, exports what include/picospec.h declares, and every
host-checkable misuse is rejected with its error code before anything is launched."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2603_19133_amd import binding
    return binding


def _declared():
    text = open(os.path.join(ROOT, "include", "picospec.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(picospec_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(B):
    names = _declared()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(B.lib, n) is not None


def test_version_limits_strerror(B):
    assert B.version() == 1000
    assert B.limit(B.LIMIT_MAX_K) == 4096 and B.limit(B.LIMIT_MAX_V) == 1 << 20 and B.limit(99) == -1
    for code in (0, -1, -2, -3, -4, -5, -77):
        assert len(B.lib.picospec_strerror(code)) > 0
    assert B.workspace_bytes(B.CALL_COMPRESS, B.F32, 4096, 151936, 4096) == 0


FAKE = 0x1000  # a non-null, 16-byte aligned address that is never dereferenced (calls fail validation first)


def _compress(B, logits=FAKE, dtype=0, ld=100, rows=2, V=100, T=1.0, k=10, top_p=0.0, outs=(FAKE,) * 5):
    return B.lib.picospec_compress(logits, dtype, ld, rows, V, T, k, top_p, *outs, None, 0, None)


def test_compress_rejects_misuse(B):
    assert _compress(B, logits=None) == B.EINVAL
    assert _compress(B, dtype=7) == B.EDTYPE
    assert _compress(B, ld=99) == B.EINVAL
    assert _compress(B, V=0) == B.EINVAL
    assert _compress(B, rows=-1) == B.EINVAL
    assert _compress(B, T=0.0) == B.EINVAL
    assert _compress(B, T=-1.0) == B.EINVAL
    assert _compress(B, T=float("nan")) == B.EINVAL
    assert _compress(B, k=0) == B.EINVAL
    assert _compress(B, k=101) == B.EINVAL
    assert _compress(B, top_p=float("nan")) == B.EINVAL
    assert _compress(B, logits=FAKE + 2) == B.EINVAL                 # fp32 base not 4-byte aligned
    assert _compress(B, V=10000, ld=10000, k=5000) == B.EUNSUPPORTED
    assert _compress(B, V=(1 << 20) + 1, ld=1 << 21) == B.EUNSUPPORTED
    for i in range(5):
        outs = [FAKE] * 5
        outs[i] = None
        assert _compress(B, outs=tuple(outs)) == B.EINVAL


def _verify(B, tgt=FAKE, dtype=0, ld=50, V=50, T=1.0, Bn=2, N=6, seq=FAKE, tok=FAKE, q=(FAKE,) * 4, k=8,
            renorm=1, qs=None, uni=FAKE, n_acc=FAKE, stats=(FAKE, FAKE), flags=FAKE):
    return B.lib.picospec_verify(tgt, dtype, ld, V, T, Bn, N, seq, tok, *q, k, renorm, qs, uni, n_acc, None, None,
                                 stats[0], stats[1], None, flags, None, 0, None)


def test_verify_rejects_misuse(B):
    assert _verify(B, tgt=None) == B.EINVAL
    assert _verify(B, dtype=2) == B.EDTYPE
    assert _verify(B, Bn=-1) == B.EINVAL
    assert _verify(B, N=-1) == B.EINVAL
    assert _verify(B, T=0.0) == B.EINVAL
    assert _verify(B, ld=49) == B.EINVAL
    assert _verify(B, renorm=2) == B.EINVAL
    assert _verify(B, seq=None) == B.EINVAL
    assert _verify(B, tok=None) == B.EINVAL
    assert _verify(B, uni=None) == B.EINVAL
    assert _verify(B, n_acc=None) == B.EINVAL
    assert _verify(B, flags=None) == B.EINVAL
    assert _verify(B, stats=(None, FAKE)) == B.EINVAL
    assert _verify(B, q=(None, FAKE, FAKE, FAKE)) == B.EINVAL       # sparse record required ...
    assert _verify(B, k=0) == B.EINVAL
    assert _verify(B, N=2 ** 31 - 1, Bn=5) == B.EINVAL               # row count overflows int32


def _residual(B, tgt=FAKE, dtype=1, ld=64, V=64, T=0.5, Bn=3, N=5, seq=FAKE, n_acc=FAKE, stats=(FAKE, FAKE),
              q=(FAKE,) * 4, k=4, renorm=1, uni=FAKE, outs=(FAKE, FAKE, FAKE)):
    return B.lib.picospec_sample_residual(tgt, dtype, ld, V, T, Bn, N, seq, n_acc, *stats, *q, k, renorm, uni, *outs,
                                          None, 0, None)


def test_sample_residual_rejects_misuse(B):
    assert _residual(B, tgt=None) == B.EINVAL
    assert _residual(B, tgt=FAKE + 1) == B.EINVAL                    # bf16 base not 2-byte aligned
    assert _residual(B, dtype=-1) == B.EDTYPE
    assert _residual(B, V=0) == B.EINVAL
    assert _residual(B, T=float("inf")) == B.EINVAL
    assert _residual(B, renorm=-1) == B.EINVAL
    assert _residual(B, n_acc=None) == B.EINVAL
    assert _residual(B, stats=(FAKE, None)) == B.EINVAL
    assert _residual(B, q=(FAKE, None, FAKE, FAKE)) == B.EINVAL
    assert _residual(B, k=0) == B.EINVAL
    assert _residual(B, outs=(None, FAKE, FAKE)) == B.EINVAL
    assert _residual(B, outs=(FAKE, FAKE, None)) == B.EINVAL


def test_sample_draft_rejects_misuse(B):
    f = B.lib.picospec_sample_draft
    assert f(None, FAKE, FAKE, FAKE, 4, 2, FAKE, FAKE, None, None) == B.EINVAL
    assert f(FAKE, FAKE, FAKE, FAKE, 0, 2, FAKE, FAKE, None, None) == B.EINVAL
    assert f(FAKE, FAKE, FAKE, FAKE, 4, -2, FAKE, FAKE, None, None) == B.EINVAL
    assert f(FAKE, FAKE, FAKE, FAKE, 4, 2, None, FAKE, None, None) == B.EINVAL
    assert f(FAKE, FAKE, FAKE, FAKE, 4, 2, FAKE, None, None, None) == B.EINVAL


def test_binding_fails_loudly_without_library(tmp_path, monkeypatch):
    """There is no CPU fallback: a missing library is an ImportError, not a silent slow path."""
    import importlib.util
    src = os.path.join(ROOT, "paper_2603_19133_amd", "binding.py")
    dst = tmp_path / "binding_copy.py"
    dst.write_text(open(src).read())
    spec = importlib.util.spec_from_file_location("binding_copy", dst)
    with pytest.raises(ImportError, match="no CPU fallback"):
        spec.loader.exec_module(importlib.util.module_from_spec(spec))


def test_downlink_calls_reject_misuse(B):
    """Host-visible misuse of the downlink calls returns an error code before any launch (no GPU needed)."""
    lib = B.lib
    f32 = 0
    # row statistics: null outputs, bad temperature
    assert lib.picospec_row_stats(FAKE, f32, 100, 2, 100, 1.0, None, FAKE, None, None) == B.EINVAL
    assert lib.picospec_row_stats(FAKE, f32, 100, 2, 100, 0.0, FAKE, FAKE, None, None) == B.EINVAL
    assert lib.picospec_row_stats(FAKE, 7, 100, 2, 100, 1.0, FAKE, FAKE, None, None) == B.EDTYPE
    # record of the rejected rows: k out of range, missing row map, k beyond the limit
    ok = dict(tgt=FAKE, dt=f32, ld=50, V=50, T=1.0, Bn=2, N=6, seq=FAKE, na=FAKE, k=8, tp=0.0, outs=(FAKE,) * 5)

    def rej(**kw):
        a = dict(ok, **kw)
        return lib.picospec_compress_rejected(a["tgt"], a["dt"], a["ld"], a["V"], a["T"], a["Bn"], a["N"], a["seq"], a["na"],
                                              a["k"], a["tp"], *a["outs"], None, 0, None)

    assert rej(k=0) == B.EINVAL and rej(k=51) == B.EINVAL and rej(seq=None) == B.EINVAL and rej(na=None) == B.EINVAL
    assert rej(outs=(FAKE, None, FAKE, FAKE, FAKE)) == B.EINVAL and rej(Bn=-1) == B.EINVAL
    assert rej(V=10000, ld=10000, k=5000) == B.EUNSUPPORTED
    # local resampling: renorm flag, null record, missing draft statistics
    okr = dict(d=FAKE, dt=f32, ld=50, V=50, T=1.0, Bn=2, N=6, seq=FAKE, na=FAKE, st=(FAKE, FAKE), rec=(FAKE,) * 4, k=8,
               rn=0, u=FAKE, outs=(FAKE,) * 3)

    def res(**kw):
        a = dict(okr, **kw)
        return lib.picospec_resample_sparse(a["d"], a["dt"], a["ld"], a["V"], a["T"], a["Bn"], a["N"], a["seq"], a["na"],
                                            *a["st"], *a["rec"], a["k"], a["rn"], a["u"], *a["outs"], None, 0, None)

    assert res(rn=2) == B.EINVAL and res(rec=(FAKE, None, FAKE, FAKE)) == B.EINVAL and res(st=(None, FAKE)) == B.EINVAL
    assert res(k=0) == B.EINVAL and res(k=5000) == B.EUNSUPPORTED and res(u=None) == B.EINVAL
    assert res(outs=(None, FAKE, FAKE)) == B.EINVAL and res(T=float("nan")) == B.EINVAL


def test_verify_range_rejects_misuse(B):
    """Host-visible misuse of the ranged verification returns an error code before any launch."""
    lib = B.lib

    def vr(Bn=2, N=6, seq=FAKE, tok=FAKE, rec=(FAKE,) * 4, k=8, rn=1, qs=None, u=FAKE, rng=(FAKE, FAKE), gmax=4,
           outs=(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE), T=1.0):
        return lib.picospec_verify_range(FAKE, 0, 50, 50, T, Bn, N, seq, tok, *rec, k, rn, qs, u, *rng, gmax, *outs, None, 0, None)

    assert vr(gmax=-1) == B.EINVAL and vr(gmax=7) == B.EINVAL and vr(Bn=70000, N=70000, gmax=1) == B.EUNSUPPORTED
    assert vr(seq=None) == B.EINVAL and vr(tok=None) == B.EINVAL and vr(rn=2) == B.EINVAL and vr(u=None) == B.EINVAL
    assert vr(rec=(FAKE, None, FAKE, FAKE)) == B.EINVAL and vr(k=0) == B.EINVAL and vr(T=0.0) == B.EINVAL
    assert vr(outs=(None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE)) == B.EINVAL
    assert vr(outs=(FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE)) == B.EINVAL


def test_round_rejects_misuse(B):
    """The one-call round checks everything the three calls it stands for check, before any launch."""
    lib = B.lib

    def rd(draft=FAKE, tgt=FAKE, dt=0, ldd=50, ldt=50, V=50, T=1.0, Bn=2, N=6, seq=FAKE, tok=FAKE, k=8, tp=0.0, rn=1,
           u=FAKE, rec=(FAKE,) * 5, ver=(FAKE,) * 7, res=(FAKE,) * 3):
        return lib.picospec_round(draft, tgt, dt, ldd, ldt, V, T, Bn, N, seq, tok, k, tp, rn, u, *rec, *ver, *res, None, 0, None)

    assert rd(draft=None) == B.EINVAL and rd(tgt=None) == B.EINVAL and rd(dt=3) == B.EDTYPE
    assert rd(ldd=49) == B.EINVAL and rd(ldt=49) == B.EINVAL and rd(V=0) == B.EINVAL
    assert rd(T=0.0) == B.EINVAL and rd(T=float("nan")) == B.EINVAL and rd(Bn=-1) == B.EINVAL and rd(N=-1) == B.EINVAL
    assert rd(seq=None) == B.EINVAL and rd(tok=None) == B.EINVAL and rd(u=None) == B.EINVAL and rd(rn=2) == B.EINVAL
    assert rd(k=0) == B.EINVAL and rd(k=51) == B.EINVAL and rd(tp=float("nan")) == B.EINVAL
    assert rd(V=10000, ldd=10000, ldt=10000, k=5000) == B.EUNSUPPORTED
    for i in range(5):
        rec = [FAKE] * 5
        rec[i] = None
        assert rd(rec=tuple(rec)) == B.EINVAL
    for i in (0, 3, 4, 6):                           # n_accept, tgt_max, tgt_sum, verify_flags are required
        ver = [FAKE] * 7
        ver[i] = None
        assert rd(ver=tuple(ver)) == B.EINVAL
    for i in (0, 2):                                 # out_tok and residual_flags are required
        res = [FAKE] * 3
        res[i] = None
        assert rd(res=tuple(res)) == B.EINVAL


def test_wire_calls_reject_misuse_and_report_sizes(B):
    """Host-visible misuse of the wire calls returns an error code before any launch; the size helpers give
    the paper's payload arithmetic (Section 3.3: 8 bytes per entry / per drafted token) plus the headers."""
    lib = B.lib
    assert B.downlink_bytes_max(1, 10, B.WIRE_FP32) == 8 + 8 + 80 and B.downlink_bytes_max(1, 10, B.WIRE_FP16) == 8 + 8 + 60
    assert B.downlink_bytes_max(3, 5, B.WIRE_BF16) == 8 + 24 + 92 and B.downlink_bytes_max(0, 7, 0) == 8
    assert B.downlink_bytes_max(1, 10, 3) == -1 and B.downlink_bytes_max(-1, 10, 0) == -1 and B.downlink_bytes_max(1, 5000, 0) == -1
    assert B.uplink_bytes(1, 6, B.WIRE_FP32) == 8 + 4 + 48 and B.uplink_bytes(1, 6, B.WIRE_FP16) == 48
    assert B.uplink_bytes(3, 7, B.WIRE_BF16) == 8 + 8 + 28 + 16 and B.uplink_bytes(2, 3, 9) == -1
    odd = C.c_void_p(0x1002)

    def pd(Bn=2, seq=FAKE, na=FAKE, tok=FAKE, rec=(FAKE, FAKE, FAKE), k=8, fmt=0, wire=FAKE, cap=4096, nb=FAKE, st=FAKE):
        return lib.picospec_pack_downlink(Bn, seq, na, tok, *rec, k, fmt, wire, cap, nb, st, None)

    assert pd(Bn=-1) == B.EINVAL and pd(fmt=3) == B.EINVAL and pd(seq=None) == B.EINVAL and pd(na=None) == B.EINVAL
    assert pd(rec=(FAKE, None, FAKE)) == B.EINVAL and pd(k=0) == B.EINVAL and pd(k=5000) == B.EUNSUPPORTED
    assert pd(wire=None) == B.EINVAL and pd(wire=odd) == B.EINVAL and pd(cap=4) == B.EINVAL
    assert pd(nb=None) == B.EINVAL and pd(st=None) == B.EINVAL

    def ud(wire=FAKE, n=64, Bn=2, k=8, outs=(FAKE,) * 6, st=FAKE):
        return lib.picospec_unpack_downlink(wire, n, Bn, k, *outs, st, None)

    assert ud(wire=None) == B.EINVAL and ud(wire=odd) == B.EINVAL and ud(n=-1) == B.EINVAL and ud(Bn=-1) == B.EINVAL
    assert ud(k=0) == B.EINVAL and ud(k=5000) == B.EUNSUPPORTED and ud(st=None) == B.EINVAL
    assert ud(outs=(FAKE, FAKE, None, FAKE, FAKE, FAKE)) == B.EINVAL

    def pu(Bn=2, N=6, seq=FAKE, tok=FAKE, q=FAKE, fmt=0, wire=FAKE, cap=4096, nb=FAKE):
        return lib.picospec_pack_uplink(Bn, N, seq, tok, q, fmt, wire, cap, nb, None)

    assert pu(Bn=-1) == B.EINVAL and pu(N=-1) == B.EINVAL and pu(fmt=-1) == B.EINVAL and pu(seq=None) == B.EINVAL
    assert pu(tok=None) == B.EINVAL and pu(q=None) == B.EINVAL and pu(wire=None) == B.EINVAL and pu(wire=odd) == B.EINVAL
    assert pu(cap=B.uplink_bytes(2, 6, 0) - 1) == B.EINVAL and pu(nb=None) == B.EINVAL

    def uu(wire=FAKE, n=64, Bn=2, nmax=6, seq=FAKE, tok=FAKE, q=FAKE, st=FAKE):
        return lib.picospec_unpack_uplink(wire, n, Bn, nmax, seq, tok, q, st, None)

    assert uu(wire=None) == B.EINVAL and uu(wire=odd) == B.EINVAL and uu(n=-1) == B.EINVAL and uu(Bn=-1) == B.EINVAL
    assert uu(nmax=-1) == B.EINVAL and uu(seq=None) == B.EINVAL and uu(tok=None) == B.EINVAL and uu(st=None) == B.EINVAL


def test_compress_kernels_keep_claimed_slots_in_registers():
    """The compress kernels issue LDS atomics by hand and read their results later (after an explicit wait); a
    register spilled in between would carry a stale value.  The generated code (cross-compiled here, no GPU needed)
    must therefore hold no scratch access between a hand-issued atomic and the wait that follows it, in any kernel;
    the kernels that run the hot path (the variants of the compress kernel, the small rounds' streaming kernel) must
    not touch scratch memory at all."""
    import subprocess
    import tempfile
    from paper_2603_19133_amd import build as bld
    if not os.path.exists(bld.HIPCC):
        pytest.skip("hipcc not found")
    src = os.path.join(bld.CSRC, "compress.hip")
    flags = [f for f in bld.FLAGS if f not in ("-shared", "-fPIC")]
    with tempfile.TemporaryDirectory() as tmp:
        asm = os.path.join(tmp, "compress.s")
        out = subprocess.run([bld.HIPCC, *flags, "-S", "--cuda-device-only", "-o", asm, src], capture_output=True, text=True)
        assert out.returncode == 0, out.stderr[-2000:]
        lines = open(asm).read().split("\n")
    kernels = {}
    name, pending, by_hand = None, False, False
    for line in lines:
        m = re.match(r"^(_ZN8picospec\S+):", line)
        if m:
            name, pending, by_hand = m.group(1), False, False
            kernels[name] = dict(atomics=0, scratch=0, in_window=0)
            continue
        if name is None:
            continue
        ins = line.strip()
        if ins.startswith(";;#ASMSTART") or ins.startswith(";;#ASMEND"):
            by_hand = ins.startswith(";;#ASMSTART")
        elif ins.startswith("s_endpgm"):
            name = None
        elif ins.startswith("ds_add_rtn") and by_hand:       # (the compiler tracks the atomics that it issues itself)
            kernels[name]["atomics"] += 1
            pending = True
        elif ins.startswith("s_waitcnt") and "lgkmcnt(0)" in ins:
            pending = False
        elif ins.startswith("scratch_"):
            kernels[name]["scratch"] += 1
            kernels[name]["in_window"] += pending
    claiming = {k: v for k, v in kernels.items() if v["atomics"] >= 8}
    hot = [k for k in claiming if "compress_kernel" in k or "round_stream_kernel" in k]
    assert len(hot) == 7 and len(claiming) == 9, sorted(claiming)      # + the two instantiations of the retry kernel
    assert all(v["in_window"] == 0 for v in claiming.values()), claiming
    assert all(claiming[k]["scratch"] == 0 for k in hot), {k: claiming[k] for k in hot}


def test_streaming_loads_stay_inside_the_row(B):
    """The row loads of the compress and residual kernels, look-ahead included, never address a byte behind the aligned
    16-byte block that holds the row's last byte, whatever the row length and its alignment: the library's own
    addressing rule (the functions the kernels use), evaluated over every lane on the host."""
    sizes = [1, 2, 3, 7, 8, 9, 63, 64, 65, 255, 256, 257, 511, 512, 513, 1000, 2047, 2048, 2049, 4095, 4096, 4097,
             8191, 8192, 8193, 16383, 16384, 16385, 16400, 32000, 32767, 32768, 32769, 65535, 65537, 128256, 151936,
             152064, (1 << 20) - 1, 1 << 20]
    for which in (B.CALL_COMPRESS, B.CALL_SAMPLE_RESIDUAL):
        for dtype, esz in ((B.F32, 4), (B.BF16, 2)):
            for V in sizes:
                for mis in range(0, 16, esz):
                    end = B.max_load_byte(which, dtype, V, mis)
                    row_bytes = V * esz
                    allowed = (mis + row_bytes + 15) // 16 * 16 - mis      # end of the last byte's aligned block
                    assert row_bytes - 15 <= end <= allowed, (which, dtype, V, mis, end, allowed)
    assert B.max_load_byte(B.CALL_VERIFY, B.F32, 100, 0) == -1
    assert B.max_load_byte(B.CALL_COMPRESS, B.BF16, 100, 3) == -1
    assert B.max_load_byte(B.CALL_COMPRESS, B.F32, 0, 0) == -1
    assert B.max_load_byte(B.CALL_COMPRESS, B.F32, (1 << 20) + 1, 0) == -1


def test_check_device_rejects_misuse(B):
    f = B.lib.picospec_check_device
    assert f(None, 1 << 16, FAKE, None) == B.EINVAL
    assert f(FAKE, 1 << 16, None, None) == B.EINVAL
    assert f(FAKE, (1 << 16) - 1, FAKE, None) == B.EINVAL          # workspace too small
    assert f(FAKE + 4, 1 << 16, FAKE, None) == B.EINVAL             # not on a 16-byte boundary


def test_probe_clock_rejects_misuse(B):
    assert B.lib.picospec_probe_clock(None, None) == B.EINVAL
    assert B.lib.picospec_probe_clock(FAKE + 4, None) == B.EINVAL
