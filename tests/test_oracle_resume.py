"""Pins of the oracle's verification over a range of draft positions (paper Section 3.2, Fast Verification: the
cloud verifies the part of a draft that is known and goes on when the rest arrives; Section 3.3 for the test
itself) against an independent dense numpy computation, and the composition of ranges against the whole."""
import numpy as np
import pytest
import scipy.special

import oracle
from paper_2603_19133_amd import workloads as W


def _round(seed, B=9, V=211, gmax=7, T=0.8):
    rng = np.random.default_rng(seed)
    g = rng.integers(0, gmax + 1, B).astype(np.int32)
    off = W.seq_offsets(g)
    N = int(off[-1])
    tgt = (rng.standard_normal((N + B, V)) * 2).astype(np.float32)
    draft = np.empty((N, V), np.float32)
    for b in range(B):
        for i in range(g[b]):
            draft[off[b] + i] = tgt[off[b] + b + i] + rng.standard_normal(V).astype(np.float32) * 0.7
    q = oracle.compress(draft, V, T, V)                      # uncompressed: qhat is the dense draft distribution
    tok, _, _ = oracle.sample_draft(q, rng.random(N, dtype=np.float32))
    uni = rng.random(N + B, dtype=np.float32)
    return dict(g=g, off=off, N=N, B=B, V=V, T=T, tgt=tgt, draft=draft, q=q, tok=tok, uni=uni)


def _dense_first_rejection(r, begin, end):
    """Textbook rule on dense distributions, written out with scipy's softmax."""
    out = np.empty(r["B"], np.int32)
    for b in range(r["B"]):
        n = end[b]
        for t in range(begin[b], end[b]):
            i, row = r["off"][b] + t, r["off"][b] + b + t
            P = scipy.special.softmax(r["tgt"][row].astype(np.float64) / r["T"])
            Q = scipy.special.softmax(r["draft"][i].astype(np.float64) / r["T"])
            x = r["tok"][i]
            if not (float(r["uni"][row]) < min(1.0, P[x] / Q[x])):
                n = t
                break
        out[b] = n
    return out


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_ranges_against_the_dense_rule(seed):
    r = _round(seed)
    rng = np.random.default_rng(100 + seed)
    end = np.array([rng.integers(0, gi + 1) for gi in r["g"]], np.int32)
    begin = np.array([rng.integers(0, e + 1) for e in end], np.int32)
    v = oracle.verify(r["tgt"], r["V"], r["T"], r["off"], r["tok"], r["q"], r["uni"], pos_begin=begin, pos_end=end)
    assert np.array_equal(v.n_accept, _dense_first_rejection(r, begin, end))
    # rows begin..end got their statistics (library log-sum-exp), nothing else was written
    for b in range(r["B"]):
        t0 = r["off"][b] + b
        for t in range(r["g"][b] + 1):
            want = scipy.special.logsumexp(r["tgt"][t0 + t].astype(np.float64) / r["T"])
            if begin[b] <= t <= end[b]:
                assert v.tgt_lse[t0 + t] == pytest.approx(want, rel=1e-12)
            else:
                assert np.isnan(v.tgt_lse[t0 + t])
            if t < r["g"][b]:
                assert np.isnan(v.p_tok[r["off"][b] + t]) == (not (begin[b] <= t < end[b]))
    # the defaults are the whole sequence
    whole = oracle.verify(r["tgt"], r["V"], r["T"], r["off"], r["tok"], r["q"], r["uni"])
    assert np.array_equal(whole.n_accept, _dense_first_rejection(r, np.zeros(r["B"], np.int32), r["g"]))


@pytest.mark.parametrize("seed", [5, 6, 7])
def test_consecutive_ranges_compose_to_the_whole(seed):
    r = _round(seed, B=12, gmax=9)
    rng = np.random.default_rng(seed)
    whole = oracle.verify(r["tgt"], r["V"], r["T"], r["off"], r["tok"], r["q"], r["uni"])
    cut1 = np.array([rng.integers(0, gi + 1) for gi in r["g"]], np.int32)
    cut2 = np.array([rng.integers(c, gi + 1) for c, gi in zip(cut1, r["g"])], np.int32)
    acc = None
    n = None
    for begin, end in ((np.zeros_like(cut1), cut1), (cut1, cut2), (cut2, r["g"])):
        acc = oracle.verify(r["tgt"], r["V"], r["T"], r["off"], r["tok"], r["q"], r["uni"], pos_begin=begin, pos_end=end, out=acc)
        part = acc.n_accept.copy()
        n = part if n is None else np.where(n < begin, n, part)      # an earlier rejection stands
    assert np.array_equal(n, whole.n_accept)
    assert np.array_equal(acc.tgt_lse, whole.tgt_lse) and np.array_equal(acc.p_tok, whole.p_tok) and np.array_equal(acc.q_tok, whole.q_tok)


def test_range_limits_are_clamped():
    r = _round(9)
    B, g = r["B"], r["g"]
    whole = oracle.verify(r["tgt"], r["V"], r["T"], r["off"], r["tok"], r["q"], r["uni"])
    wide = oracle.verify(r["tgt"], r["V"], r["T"], r["off"], r["tok"], r["q"], r["uni"],
                         pos_begin=np.full(B, -3, np.int32), pos_end=g + 5)
    assert np.array_equal(wide.n_accept, whole.n_accept) and np.array_equal(wide.tgt_lse, whole.tgt_lse)
    crossed = oracle.verify(r["tgt"], r["V"], r["T"], r["off"], r["tok"], r["q"], r["uni"],
                            pos_begin=g + 2, pos_end=np.minimum(g, 1).astype(np.int32))
    assert np.array_equal(crossed.n_accept, np.minimum(g, 1))          # an empty range: nothing rejected in it
    assert np.all(np.isnan(crossed.p_tok))
