"""GPU parity of the verification over a range of draft positions (Section 3.2, Fast Verification; Section 3.3
for the acceptance test) through the C ABI against the oracle, and the composition of consecutive ranges."""
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


def _setup(pu, ps, gpu, r, k):
    w = r.workload
    q = oracle.compress(r.draft_logits, w.V, w.T, k)
    tok, _, _ = oracle.sample_draft(q, r.draft_uniforms)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(gpu)
    gq = ps.compress(pu.to_device(r.draft_logits, gpu), w.V, w.T, k)
    return q, tok, gq, pu.to_device(r.tgt_logits, gpu), d(r.seq_off), d(tok), d(r.uniforms), d


def _compare_range(pu, r, g, o, begin, end):
    """Entries of the range against the oracle's; sequences whose decision is knife-edge in the oracle are skipped."""
    off = r.seq_off
    p_tok, q_tok, lse = pu.n(g.p_tok), pu.n(g.q_tok), pu.n(g.tgt_lse)
    n_acc = pu.n(g.n_accept)
    for b in range(r.B):
        d0, t0 = off[b], off[b] + b
        sl = slice(d0 + begin[b], d0 + end[b])
        pu.assert_close(p_tok[sl], o.p_tok[sl], pu.RTOL, "p_tok", atol=1e-30)
        pu.assert_close(q_tok[sl], o.q_tok[sl], pu.RTOL, "q_tok", atol=1e-30)
        rows = slice(t0 + begin[b], t0 + end[b] + 1)
        pu.assert_close(lse[rows], o.tgt_lse[rows], pu.RTOL_LSE, "tgt_lse", atol=2e-6)
        if o.margin[sl].min(initial=np.inf) >= pu.ACCEPT_MARGIN:
            assert n_acc[b] == o.n_accept[b], (b, begin[b], end[b])
    assert np.array_equal(pu.n(g.flags).astype(np.uint32), o.flags)


@pytest.mark.parametrize("name,scale,k", [("cfg1", dict(B=6), 64), ("cfg2", dict(B=8), 256), ("cfg5", dict(B=24, V=20011, k=512), 512)])
def test_ranges_match_the_oracle_and_compose(gpu, pu, ps, name, scale, k):
    _announce("verify_range", name, k)
    w = W.WORKLOADS[name].scaled(**scale)
    _ranges_case(pu, ps, gpu, W.build_round(w, 0), k, 3)


def _ranges_case(pu, ps, gpu, r, k, seed):
    """Three consecutive random ranges per sequence: each against the oracle, together against the whole call."""
    w = r.workload
    q, tok, gq, tgt, seq_off, dtok, uni, d = _setup(pu, ps, gpu, r, k)
    g = np.diff(r.seq_off).astype(np.int32)
    gmax = int(g.max(initial=0))
    rng = np.random.default_rng(seed)
    cut1 = np.array([rng.integers(0, gi + 1) for gi in g], np.int32)
    cut2 = np.array([rng.integers(c, gi + 1) for c, gi in zip(cut1, g)], np.int32)
    whole_o = oracle.verify(r.tgt_logits, w.V, w.T, r.seq_off, tok, q, r.uniforms)
    whole_g = ps.verify(tgt, w.V, w.T, seq_off, r.N, dtok, gq, uni)
    acc_g = ps.alloc_verified(r.B, r.N, gpu)
    for t in (acc_g.p_tok, acc_g.q_tok, acc_g.tgt_max, acc_g.tgt_sum, acc_g.tgt_lse):
        t.fill_(-5.0)
    acc_o, n_g = None, None
    for begin, end in ((np.zeros_like(cut1), cut1), (cut1, cut2), (cut2, g)):
        acc_o = oracle.verify(r.tgt_logits, w.V, w.T, r.seq_off, tok, q, r.uniforms, pos_begin=begin, pos_end=end, out=acc_o)
        ps.verify_range(tgt, w.V, w.T, seq_off, r.N, dtok, gq, uni, d(begin), d(end), gmax, out=acc_g)
        torch.cuda.synchronize()
        _compare_range(pu, r, acc_g, acc_o, begin, end)
        part = pu.n(acc_g.n_accept).copy()
        n_g = part if n_g is None else np.where(n_g < begin, n_g, part)
    # the three ranges together are the whole call, bit for bit (same kernels, same rows)
    assert np.array_equal(n_g, pu.n(whole_g.n_accept))
    for a, b in ((acc_g.p_tok, whole_g.p_tok), (acc_g.q_tok, whole_g.q_tok), (acc_g.tgt_max, whole_g.tgt_max),
                 (acc_g.tgt_sum, whole_g.tgt_sum), (acc_g.tgt_lse, whole_g.tgt_lse)):
        assert torch.equal(a, b)
    assert np.array_equal(acc_o.tgt_lse, whole_o.tgt_lse) and np.array_equal(acc_o.p_tok, whole_o.p_tok)


def test_defaults_untouched_entries_and_clamping(gpu, pu, ps):
    _announce("verify_range defaults")
    w = W.WORKLOADS["cfg2"].scaled(B=5)
    r = W.build_round(w, 0)
    q, tok, gq, tgt, seq_off, dtok, uni, d = _setup(pu, ps, gpu, r, 256)
    g = np.diff(r.seq_off).astype(np.int32)
    gmax = int(g.max())
    whole = ps.verify(tgt, w.V, w.T, seq_off, r.N, dtok, gq, uni)
    both_null = ps.verify_range(tgt, w.V, w.T, seq_off, r.N, dtok, gq, uni, None, None, gmax)
    torch.cuda.synchronize()
    assert torch.equal(both_null.n_accept, whole.n_accept) and torch.equal(both_null.tgt_lse, whole.tgt_lse)
    assert torch.equal(both_null.p_tok, whole.p_tok) and torch.equal(both_null.flags, whole.flags)
    # a range in the middle: everything outside keeps the sentinel
    begin, end = np.minimum(g, 2).astype(np.int32), np.minimum(g, 5).astype(np.int32)
    out = ps.alloc_verified(r.B, r.N, gpu)
    for t in (out.p_tok, out.q_tok, out.tgt_max, out.tgt_sum, out.tgt_lse):
        t.fill_(-5.0)
    ps.verify_range(tgt, w.V, w.T, seq_off, r.N, dtok, gq, uni, d(begin), d(end), gmax, out=out)
    torch.cuda.synchronize()
    p, lse = pu.n(out.p_tok), pu.n(out.tgt_lse)
    for b in range(r.B):
        d0, t0 = r.seq_off[b], r.seq_off[b] + b
        for t in range(g[b] + 1):
            assert (lse[t0 + t] != -5.0) == (begin[b] <= t <= end[b])
            if t < g[b]:
                assert (p[d0 + t] != -5.0) == (begin[b] <= t < end[b])
    # limits outside the sequence are clamped and flagged; an empty range rejects nothing
    o = oracle.verify(r.tgt_logits, w.V, w.T, r.seq_off, tok, q, r.uniforms, pos_begin=np.full(r.B, -2, np.int32), pos_end=g + 3)
    wide = ps.verify_range(tgt, w.V, w.T, seq_off, r.N, dtok, gq, uni, d(np.full(r.B, -2, np.int32)), d(g + 3), gmax)
    torch.cuda.synchronize()
    assert np.array_equal(pu.n(wide.n_accept), o.n_accept) and bool(((wide.flags & ps.FLAG_BAD_INPUT) != 0).all())
    empty = ps.verify_range(tgt, w.V, w.T, seq_off, r.N, dtok, gq, uni, d(np.minimum(g, 1).astype(np.int32)),
                            d(np.minimum(g, 1).astype(np.int32)), gmax)
    torch.cuda.synchronize()
    assert np.array_equal(pu.n(empty.n_accept), np.minimum(g, 1)) and bool((empty.flags == 0).all())
    # host-visible misuse
    with pytest.raises(ps.PicoSpecError):
        ps.verify_range(tgt, w.V, w.T, seq_off, r.N, dtok, gq, uni, None, None, -1)
    with pytest.raises(ps.PicoSpecError):
        ps.verify_range(tgt, w.V, w.T, seq_off, r.N, dtok, gq, uni, None, None, r.N + 1)
