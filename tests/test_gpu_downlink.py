"""GPU parity of the paper-literal downlink (Section 3.3, Eq. 4): the Top-K record of the target row at
the rejected position, and the edge's local resampling against its dense draft distribution, through
the C ABI against the oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_19133_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ps():
    from paper_2603_19133_amd import binding
    return binding


@pytest.fixture(scope="module")
def pu():
    import parity_util
    return parity_util


def _announce(*a):
    print("[case]", *a, flush=True)


def _downlink(pu, ps, gpu, r, k, renorm, n_accept=None, top_p=0.0, strict=True):
    """Oracle and library on one round: verify with the scalar uplink, record of the rejected row, local resampling."""
    w = r.workload
    # the drafter's tokens and scalar q_i (edge side: dense draft distribution, here through a full-support record)
    qd = oracle.compress(r.draft_logits, w.V, w.T, min(w.V, 4096))
    tok, slot, _ = oracle.sample_draft(qd, r.draft_uniforms)
    q_scalar = (qd.prob[np.arange(r.N), slot] / qd.mass).astype(np.float64) if r.N else np.zeros(0)
    ov = oracle.verify(r.tgt_logits, w.V, w.T, r.seq_off, tok, qd, r.uniforms, renorm=1, q_scalar=q_scalar)
    na = ov.n_accept if n_accept is None else np.asarray(n_accept, np.int32)
    orec = oracle.compress_rejected(r.tgt_logits, w.V, w.T, r.seq_off, na, k, top_p)
    ores = oracle.resample_sparse(r.draft_logits, w.V, w.T, r.seq_off, na, orec, r.uniforms, renorm)

    draft, tgt = pu.to_device(r.draft_logits, gpu), pu.to_device(r.tgt_logits, gpu)
    seq_off = torch.from_numpy(r.seq_off).to(gpu)
    uni = torch.from_numpy(r.uniforms).to(gpu)
    na_d = torch.from_numpy(na).to(gpu)
    grec = ps.compress_rejected(tgt, w.V, w.T, seq_off, r.N, na_d, k, top_p)
    dmax, dsum, dlse = ps.row_stats(draft, w.V, w.T)
    gres = ps.resample_sparse(draft, w.V, w.T, seq_off, r.N, na_d, dmax, dsum, grec, uni, renorm)
    torch.cuda.synchronize()

    st = pu.compare_compress(grec, orec, top_p)
    if r.N:
        olse = oracle.compress(r.draft_logits, w.V, w.T, 1).lse
        pu.assert_close(pu.n(dlse), olse, pu.RTOL_LSE, "draft lse", atol=2e-6)
    # strict: relative tolerance only.  Otherwise (rounds with peaked or identical rows) a sequence whose ORACLE residual
    # mass lies below PEAKED_R carries the absolute term RESID_ATOL, and a residual mass within it of zero is not
    # compared for emptiness (flag, fallback draw from the record): in exact arithmetic such a position is never rejected
    atol_b = np.zeros(r.B) if strict else np.where(ores.resid_mass < pu.PEAKED_R, pu.RESID_ATOL, 0.0)
    undecided = np.zeros(r.B, bool) if strict else ores.resid_mass <= pu.RESID_ATOL
    assert (pu.n(gres.flags).astype(np.uint32) == ores.flags)[~undecided].all()
    st["resid_mass"] = pu.assert_close(pu.n(gres.resid_mass), ores.resid_mass, pu.RTOL, "resid_mass", atol=atol_b)
    same = pu.n(gres.out_tok) == ores.out_tok
    knife = (ores.cdf_margin < pu.CDF_MARGIN + atol_b / np.maximum(ores.resid_mass, 1e-300)) | undecided
    excl = set(st["topp_excluded"])
    for b in np.nonzero(~same)[0]:
        assert knife[b] or b in excl, (b, pu.n(gres.out_tok)[b], ores.out_tok[b], ores.cdf_margin[b])
    st["mismatch_draw"] = int((~same & ~undecided).sum())
    assert st["mismatch_draw"] <= max(1, r.B // 50)
    return st, ores


CASES = [("cfg1", {}, 64), ("cfg2", {}, 256), ("cfg3", {"B": 6}, 1024), ("cfg4", {"B": 3}, 4096), ("cfg5", {"B": 10}, 2048),
         ("cfg2", {}, 10), ("cfg3", {"B": 6}, 10)]


@pytest.mark.parametrize("renorm", [0, 1])
@pytest.mark.parametrize("name,scale,k", CASES)
def test_downlink_round_matches_oracle(gpu, pu, ps, name, scale, k, renorm):
    w = W.WORKLOADS[name]
    if scale:
        w = w.scaled(**scale)
    _announce("downlink round", name, scale, "K", k, "renorm", renorm)
    r = W.build_round(w, 0)
    st, _ = _downlink(pu, ps, gpu, r, k, renorm)
    print("[stats]", name, {a: b for a, b in st.items() if a != "topp_excluded"}, flush=True)


def _small_round(rng, V, B=12, gmax=5, dtype="f32", same=False):
    g = rng.integers(0, gmax + 1, B).astype(np.int32)
    off = W.seq_offsets(g)
    N = int(off[-1])
    tgt = (rng.standard_normal((N + B, V)) * 2.5).astype(np.float32)
    draft = np.empty((max(N, 1), V), np.float32)[:N] if N else np.zeros((0, V), np.float32)
    for b in range(B):
        for i in range(g[b]):
            draft[off[b] + i] = tgt[off[b] + b + i] + (0 if same else rng.standard_normal(V).astype(np.float32))
    if dtype == "bf16":
        tgt, draft = W.to_bf16_bits(tgt), W.to_bf16_bits(draft)
    w = W.Workload("downlink", 77, B, 0, gmax, V, dtype, 0.9, min(V, 64), 0.0, 1, "custom")
    return W.Round(w, 0, np.arange(B), off, np.ascontiguousarray(draft), tgt, rng.random(N + B, dtype=np.float32),
                   rng.random(N, dtype=np.float32)), g


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_downlink_small_ragged_every_position(gpu, pu, ps, dtype):
    """Every first-rejection index 0..gamma_b (bonus included), K = V (exact) and K < V, odd sizes."""
    _announce("downlink ragged", dtype)
    rng = np.random.default_rng(5)
    for V, k in ((97, 97), (97, 7), (1031, 100), (5000, 4096)):
        r, g = _small_round(rng, V, dtype=dtype)
        for shift in range(0, 6):
            na = np.minimum(g, shift).astype(np.int32)
            for renorm in (0, 1):
                _downlink(pu, ps, gpu, r, k, renorm, n_accept=na, strict=False)


def test_downlink_empty_residual_and_bad_inputs(gpu, pu, ps):
    _announce("downlink empty residual / bad inputs")
    rng = np.random.default_rng(9)
    r, g = _small_round(rng, 300, same=True)
    na = np.maximum(np.minimum(g - 1, 2), 0).astype(np.int32)
    w = r.workload
    draft, tgt = pu.to_device(r.draft_logits, gpu), pu.to_device(r.tgt_logits, gpu)
    seq_off = torch.from_numpy(r.seq_off).to(gpu)
    uni = torch.from_numpy(r.uniforms).to(gpu)
    na_d = torch.from_numpy(na).to(gpu)
    dmax, dsum, _ = ps.row_stats(draft, 300, w.T)
    # (a) draft == target, K = V: P and Q agree exactly in the oracle (flagged); on the GPU they agree up to fp32
    #     rounding, so either the flag is set or R is a rounding residue: both are legitimate
    orec = oracle.compress_rejected(r.tgt_logits, 300, w.T, r.seq_off, na, 300)
    ores = oracle.resample_sparse(r.draft_logits, 300, w.T, r.seq_off, na, orec, r.uniforms, 0)
    grec = ps.compress_rejected(tgt, 300, w.T, seq_off, r.N, na_d, 300)
    gres = ps.resample_sparse(draft, 300, w.T, seq_off, r.N, na_d, dmax, dsum, grec, uni, 0)
    torch.cuda.synchronize()
    for b in range(r.B):
        if na[b] < g[b]:
            assert ores.flags[b] & 4
            assert float(pu.n(gres.resid_mass)[b]) < 1e-5
    # (b) the flagged branch, deterministically: a record whose values are half of P lies below Q everywhere
    orec.prob *= 0.5
    orec.mass *= 0.5
    ores = oracle.resample_sparse(r.draft_logits, 300, w.T, r.seq_off, na, orec, r.uniforms, 0)
    half = ps.Compressed(torch.from_numpy(orec.idx).to(gpu), torch.from_numpy(orec.prob.astype(np.float32)).to(gpu),
                         torch.from_numpy(orec.count).to(gpu), torch.from_numpy(orec.mass.astype(np.float32)).to(gpu),
                         torch.from_numpy(orec.lse.astype(np.float32)).to(gpu), 300)
    gres = ps.resample_sparse(draft, 300, w.T, seq_off, r.N, na_d, dmax, dsum, half, uni, 0)
    torch.cuda.synchronize()
    for b in range(r.B):
        if na[b] < g[b]:
            assert ores.flags[b] & 4 and pu.n(gres.flags)[b] & 4 and pu.n(gres.resid_mass)[b] == 0.0
            assert pu.n(gres.out_tok)[b] == ores.out_tok[b] or ores.cdf_margin[b] < pu.CDF_MARGIN
    # n_accept outside 0..gamma_b: clamped and flagged, nothing faults
    bad = torch.from_numpy(np.where(np.arange(r.B) % 2 == 0, -3, 99).astype(np.int32)).to(gpu)
    rec = ps.compress_rejected(tgt, 300, 0.9, seq_off, r.N, bad, 50)
    res = ps.resample_sparse(draft, 300, 0.9, seq_off, r.N, bad, dmax, dsum, rec, uni, 0)
    torch.cuda.synchronize()
    assert (pu.n(res.flags) & 8).all()
    tok = pu.n(res.out_tok)
    assert ((tok >= 0) & (tok < 300)).all()
    clamped = np.where(np.arange(r.B) % 2 == 0, 0, g).astype(np.int32)
    want = oracle.compress_rejected(r.tgt_logits, 300, 0.9, r.seq_off, clamped, 50)
    assert (pu.n(rec.idx) == want.idx).all()
    # empty batch
    e32 = torch.zeros(1, dtype=torch.int32, device=gpu)
    rec0 = ps.compress_rejected(tgt[:0], 300, 0.9, e32, 0, e32[:0], 10)
    res0 = ps.resample_sparse(draft[:0], 300, 0.9, e32, 0, e32[:0], dmax[:0], dsum[:0], rec0, uni[:0], 0)
    torch.cuda.synchronize()
    assert rec0.idx.shape[0] == 0 and res0.out_tok.shape[0] == 0
