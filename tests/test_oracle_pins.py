"""Pins of the CPU oracle against what the paper and the mathematics fix (CPU only).

Each test compares the oracle with something that is not the oracle: a library routine, a dense
textbook implementation written independently in numpy, a closed form, a statistical law, a figure
the paper prints, or brute force on a tiny vocabulary.
"""
import math
import os

import numpy as np
import pytest
import scipy.special
import scipy.stats

import oracle
from paper_2603_19133_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append(line.split())
    return rows


def _softmax64(z, T):
    return scipy.special.softmax(np.asarray(z, np.float64) / T, axis=-1)


# ---------------------------------------------------------------- log-sum-exp / probabilities

@pytest.mark.parametrize("T", [1.0, 0.7, 2.5])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_lse_and_probs_match_library_softmax(T, dtype):
    rng = np.random.default_rng(1)
    z = (rng.standard_normal((5, 1000)) * 4).astype(np.float32)
    stored = z if dtype == "f32" else W.to_bf16_bits(z)
    exact = z if dtype == "f32" else W.bf16_bits_to_f32(stored)
    q = oracle.compress(stored, 1000, T, 17)
    ref_lse = scipy.special.logsumexp(exact.astype(np.float64) / T, axis=1)
    np.testing.assert_allclose(q.lse, ref_lse, rtol=1e-13)
    P = _softmax64(exact, T)
    for r in range(5):
        np.testing.assert_allclose(q.prob[r], P[r, q.idx[r]], rtol=1e-12)
        np.testing.assert_allclose(q.mass[r], P[r, q.idx[r]].sum(), rtol=1e-12)


def test_bf16_widening_is_exact():
    bits = np.array([[0x3F80, 0xC000, 0x0000, 0x8000, 0x4049, 0xFF80]], np.uint16)  # 1,-2,0,-0,3.140625,-inf
    q = oracle.compress(bits, 6, 1.0, 6)
    assert list(q.idx[0]) == [4, 0, 2, 3, 1, 5]   # 0 and -0 tie -> lower index first; -inf last
    assert q.prob[0, 5] == 0.0
    np.testing.assert_allclose(q.lse[0], math.log(math.exp(3.140625) + math.e + 2 + math.exp(-2)), rtol=1e-14)


# ---------------------------------------------------------------- top-k set and order

def _lexsort_topk(z, k):
    z = np.asarray(z, np.float64)
    return np.lexsort((np.arange(z.shape[0]), -z))[:k]


@pytest.mark.parametrize("k", [1, 7, 64, 500])
def test_topk_matches_lexsort_random_and_tied(k):
    rng = np.random.default_rng(2)
    rows = [rng.standard_normal(500).astype(np.float32),
            rng.integers(-3, 4, 500).astype(np.float32),           # heavy ties
            np.zeros(500, np.float32),                              # all equal -> 0..k-1
            np.where(rng.random(500) < 0.5, -np.inf, rng.standard_normal(500)).astype(np.float32)]
    z = np.stack(rows)
    q = oracle.compress(z, 500, 1.0, k)
    for r in range(z.shape[0]):
        assert list(q.idx[r]) == list(_lexsort_topk(z[r], k)), r
    assert list(q.idx[2]) == list(range(k))
    assert (q.count == k).all()


def test_topk_bf16_ties_lower_index_wins():
    rng = np.random.default_rng(3)
    z = (rng.standard_normal((3, 4096)) * 2).astype(np.float32)
    bits = W.to_bf16_bits(z)
    exact = W.bf16_bits_to_f32(bits)
    assert len(np.unique(exact[0])) < 2000   # the rounding really does create ties
    q = oracle.compress(bits, 4096, 0.9, 300)
    for r in range(3):
        assert list(q.idx[r]) == list(_lexsort_topk(exact[r], 300))


def test_selection_does_not_depend_on_temperature():
    rng = np.random.default_rng(4)
    z = rng.standard_normal((2, 300)).astype(np.float32)
    a, b = oracle.compress(z, 300, 0.3, 40), oracle.compress(z, 300, 3.0, 40)
    assert (a.idx == b.idx).all()


def test_row_stride_is_respected():
    rng = np.random.default_rng(5)
    z = rng.standard_normal((4, 100)).astype(np.float32)
    q = oracle.compress(z, 60, 1.0, 10)     # ld = 100 > V = 60
    for r in range(4):
        assert list(q.idx[r]) == list(_lexsort_topk(z[r, :60], 10))
        np.testing.assert_allclose(q.lse[r], scipy.special.logsumexp(z[r, :60].astype(np.float64)), rtol=1e-13)


# ---------------------------------------------------------------- top-p count rule (workload setting, not in the paper)

@pytest.mark.parametrize("tau,k", [(0.5, 50), (0.9, 50), (0.95, 8), (0.999, 200)])
def test_top_p_count_matches_numpy_cumsum(tau, k):
    rng = np.random.default_rng(6)
    z = (rng.standard_normal((6, 200)) * 3).astype(np.float32)
    q = oracle.compress(z, 200, 1.0, k, top_p=tau)
    P = _softmax64(z, 1.0)
    for r in range(6):
        order = _lexsort_topk(z[r], 200)
        cum = np.cumsum(P[r, order])
        n = int(np.searchsorted(cum, tau, side="left")) + 1      # first n with cum_n >= tau
        c = min(n, k)
        assert q.count[r] == c
        assert list(q.idx[r, :c]) == list(order[:c])
        assert (q.idx[r, c:] == -1).all() and (q.prob[r, c:] == 0).all()
        np.testing.assert_allclose(q.mass[r], cum[c - 1], rtol=1e-12)


# ---------------------------------------------------------------- k = V reduces to textbook speculative sampling

def _textbook_round(draft, tgt, T, seq_off, tok, uniforms):
    """Dense standard speculative sampling, written without reference to the oracle's code."""
    B = len(seq_off) - 1
    n_acc, out = np.zeros(B, np.int64), np.zeros(B, np.int64)
    for b in range(B):
        g = seq_off[b + 1] - seq_off[b]
        d0, t0 = seq_off[b], seq_off[b] + b
        j = g
        for i in range(g):
            p = _softmax64(tgt[t0 + i], T)
            q = _softmax64(draft[d0 + i], T)
            x = tok[d0 + i]
            if not uniforms[t0 + i] < min(1.0, p[x] / q[x]):
                j = i
                break
        p = _softmax64(tgt[t0 + j], T)
        res = np.maximum(0.0, p - _softmax64(draft[d0 + j], T)) if j < g else p
        cdf = np.cumsum(res)
        out[b] = np.searchsorted(cdf, np.float64(uniforms[t0 + g]) * cdf[-1], side="right")
        n_acc[b] = j
    return n_acc, out


@pytest.mark.parametrize("renorm", [0, 1])
def test_uncompressed_equals_textbook_speculative_sampling(renorm):
    rng = np.random.default_rng(7)
    V, T = 97, 0.8
    g = np.array([4, 1, 0, 6, 3, 5, 2, 4, 4, 4], np.int32)
    off = W.seq_offsets(g)
    N, B = int(off[-1]), len(g)
    tgt = (rng.standard_normal((N + B, V)) * 2).astype(np.float32)
    draft = np.empty((N, V), np.float32)
    for b in range(B):
        for i in range(g[b]):
            draft[off[b] + i] = tgt[off[b] + b + i] + rng.standard_normal(V).astype(np.float32) * 0.7
    uni = rng.random(N + B, dtype=np.float32)
    q = oracle.compress(draft, V, T, V)
    tok, _, _ = oracle.sample_draft(q, rng.random(N, dtype=np.float32))
    v = oracle.verify(tgt, V, T, off, tok, q, uni, renorm=renorm)
    r = oracle.sample_residual(tgt, V, T, off, v.n_accept, v.tgt_lse, q, uni, renorm=renorm)
    assert v.margin.min() > 1e-9 and r.cdf_margin.min() > 1e-9      # decisions are not knife-edge
    n_acc, out = _textbook_round(draft, tgt, T, off, tok, uni)
    assert list(v.n_accept) == list(n_acc)
    assert list(r.out_tok) == list(out)
    assert 0 < v.n_accept.sum() < N                                  # both outcomes occur
    np.testing.assert_allclose(q.mass, 1.0, rtol=1e-12)
    # scalar-q uplink (the edge's recorded q_i) gives the same decisions as the sparse lookup
    v2 = oracle.verify(tgt, V, T, off, tok, None, uni, q_scalar=v.q_tok)
    assert list(v2.n_accept) == list(v.n_accept)


def test_identical_distributions_accept_everything():
    rng = np.random.default_rng(8)
    V, g = 200, np.array([5, 3, 8], np.int32)
    off = W.seq_offsets(g)
    N, B = int(off[-1]), 3
    tgt = (rng.standard_normal((N + B, V)) * 3).astype(np.float32)
    draft = np.concatenate([tgt[off[b] + b: off[b] + b + g[b]] for b in range(B)])
    uni = rng.random(N + B, dtype=np.float32)
    uni[::2] = np.float32(1.0) - np.float32(2.0 ** -24)              # largest fp32 below 1 still accepts
    q = oracle.compress(draft, V, 1.0, V)
    tok, _, _ = oracle.sample_draft(q, rng.random(N, dtype=np.float32))
    v = oracle.verify(tgt, V, 1.0, off, tok, q, uni)
    assert list(v.n_accept) == list(g)
    np.testing.assert_allclose(v.p_tok, v.q_tok, rtol=1e-12)
    r = oracle.sample_residual(tgt, V, 1.0, off, v.n_accept, v.tgt_lse, q, uni)
    for b in range(B):                                               # bonus token ~ P_gamma by inverse CDF
        p = _softmax64(tgt[off[b + 1] + b], 1.0)
        cdf = np.cumsum(p)
        assert r.out_tok[b] == np.searchsorted(cdf, np.float64(uni[off[b + 1] + b]) * cdf[-1], side="right")
    np.testing.assert_allclose(r.resid_mass, 1.0, rtol=1e-12)


# ---------------------------------------------------------------- exactness of the emitted token (chi-square, V = 8)

def _emit_first_token(V, k, renorm, n_draws, seed, T=1.0):
    rng = np.random.default_rng(seed)
    zt = (rng.standard_normal(V) * 1.5).astype(np.float32)
    zd = (zt + rng.standard_normal(V) * 1.0).astype(np.float32)
    tgt = np.tile(zt, (2 * n_draws, 1))
    draft = np.tile(zd, (n_draws, 1))
    off = np.arange(n_draws + 1, dtype=np.int32)                    # gamma = 1 everywhere
    q = oracle.compress(draft, V, T, k)
    tok, _, _ = oracle.sample_draft(q, rng.random(n_draws, dtype=np.float32))
    uni = rng.random(2 * n_draws, dtype=np.float32)
    v = oracle.verify(tgt, V, T, off, tok, q, uni, renorm=renorm)
    r = oracle.sample_residual(tgt, V, T, off, v.n_accept, v.tgt_lse, q, uni, renorm=renorm)
    emitted = np.where(v.n_accept == 1, tok, r.out_tok)
    return emitted, _softmax64(zt, T), v, r


@pytest.mark.parametrize("k,renorm", [(8, 1), (8, 0), (3, 1), (5, 1)])
def test_emitted_token_follows_target_distribution(k, renorm):
    n = 200_000
    emitted, p, _, _ = _emit_first_token(8, k, renorm, n, seed=100 + k)
    obs = np.bincount(emitted, minlength=8)
    chi = scipy.stats.chisquare(obs, p * n)
    assert chi.pvalue > 1e-3, (chi, obs, p * n)


def test_unrenormalised_truncated_draft_is_biased_negative_control():
    """With k < V and qhat = raw prob the test uses a q the token was not drawn from: detectably biased."""
    n = 200_000
    emitted, p, _, _ = _emit_first_token(8, 3, 0, n, seed=103)
    obs = np.bincount(emitted, minlength=8)
    assert scipy.stats.chisquare(obs, p * n).pvalue < 1e-6


def test_acceptance_rate_and_residual_mass_closed_form():
    n = 100_000
    _, p, v, r = _emit_first_token(8, 4, 1, n, seed=11)
    # closed form R = 1 - sum over support of min(P, qhat); acceptance probability = 1 - R
    rej = v.n_accept == 0
    R = r.resid_mass[rej][0]
    assert np.allclose(r.resid_mass[rej], R, rtol=1e-12)
    rng = np.random.default_rng(11)
    zt = (rng.standard_normal(8) * 1.5).astype(np.float32)
    zd = (zt + rng.standard_normal(8) * 1.0).astype(np.float32)
    qd = _softmax64(zd, 1.0)
    sup = np.argsort(-qd)[:4]
    qhat = qd[sup] / qd[sup].sum()
    R_closed = 1.0 - np.minimum(p[sup], qhat).sum()
    np.testing.assert_allclose(R, R_closed, rtol=1e-10)
    acc = 1.0 - rej.mean()
    assert abs(acc - (1.0 - R_closed)) < 5 * math.sqrt(R_closed * (1 - R_closed) / n)


def test_expected_generated_length_matches_eq5():
    """Eq. 5 (Section 3.4): with a constant per-token acceptance rate alpha the tokens produced per
    cycle without the bonus, min(n_accept + 1, gamma), average to (1 - alpha^gamma)/(1 - alpha)."""
    for a, g, el in _golden("eq5_expected_length.txt"):
        a, g, el = float(a), int(g), float(el)
        assert abs((1 - a ** g) / (1 - a) - el) < 1e-6
    rng = np.random.default_rng(12)
    V, g, B = 8, 4, 50_000
    zt = (rng.standard_normal(V) * 1.5).astype(np.float32)
    zd = (zt + rng.standard_normal(V) * 0.8).astype(np.float32)
    p, qd = _softmax64(zt, 1.0), _softmax64(zd, 1.0)
    alpha = np.minimum(p, qd).sum()
    off = (np.arange(B + 1) * g).astype(np.int32)
    tgt = np.tile(zt, (B * (g + 1), 1))
    draft = np.tile(zd, (B * g, 1))
    q = oracle.compress(draft, V, 1.0, V)
    tok, _, _ = oracle.sample_draft(q, rng.random(B * g, dtype=np.float32))
    v = oracle.verify(tgt, V, 1.0, off, tok, q, rng.random(B * (g + 1), dtype=np.float32))
    got = np.minimum(v.n_accept + 1, g).mean()
    want = (1 - alpha ** g) / (1 - alpha)
    assert abs(got - want) < 0.02, (got, want)
    # full geometric law of the first rejection index
    for j in range(g):
        assert abs((v.n_accept == j).mean() - alpha ** j * (1 - alpha)) < 0.01


# ---------------------------------------------------------------- record layout / payload figures printed in the paper

def test_sparse_record_payload_sizes():
    gold = {k: int(v) for k, v in _golden("payload_sizes.txt")}
    rec = oracle.record_bytes()
    assert rec == 8
    assert gold["example_K"] * rec < gold["sparse_payload_max_bytes"]
    dense = gold["vocab_llama"] * 4
    assert abs(dense - gold["dense_payload_approx_bytes"]) / gold["dense_payload_approx_bytes"] < 0.05
    assert dense / (gold["example_K"] * rec) > 1000                  # "over three orders of magnitude"
    assert gold["default_gamma"] * (4 + 4) < gold["uplink_payload_max_bytes"]


# ---------------------------------------------------------------- brute force on tiny vocabularies

def _brute_round(draft, tgt, T, k, tok, u_acc, u_res, renorm):
    """One sequence, pure Python floats, straight from the definitions."""
    def softmax(z):
        y = [float(v) / T for v in z]
        m = max(y)
        e = [math.exp(v - m) for v in y]
        s = sum(e)
        return [v / s for v in e]
    g = len(draft)
    j = g
    for i in range(g):
        qd = softmax(draft[i])
        order = sorted(range(len(qd)), key=lambda x: (-float(draft[i][x]), x))[:k]
        mass = sum(qd[x] for x in order)
        p = softmax(tgt[i])
        x = tok[i]
        qh = (qd[x] / mass if renorm else qd[x]) if x in order else 0.0
        ratio = p[x] / qh if qh > 0 else math.inf
        if not u_acc[i] < min(1.0, ratio):
            j = i
            break
    p = softmax(tgt[j])
    res = list(p)
    if j < g:
        qd = softmax(draft[j])
        order = sorted(range(len(qd)), key=lambda x: (-float(draft[j][x]), x))[:k]
        mass = sum(qd[x] for x in order)
        for x in order:
            res[x] = max(0.0, p[x] - (qd[x] / mass if renorm else qd[x]))
    R = sum(res)
    c, acc, pick = u_res * R, 0.0, None
    for x, rv in enumerate(res):
        acc += rv
        if acc > c:
            pick = x
            break
    return j, pick, R


@pytest.mark.parametrize("seed", range(12))
def test_brute_force_tiny_vocab(seed):
    rng = np.random.default_rng(1000 + seed)
    V = int(rng.integers(2, 13))
    k = int(rng.integers(1, V + 1))
    g = int(rng.integers(1, 5))
    renorm = int(seed % 2)
    T = float(rng.choice([0.5, 1.0, 1.7]))
    tgt = rng.integers(-4, 5, (g + 1, V)).astype(np.float32) * 0.5   # coarse grid: ties are common
    draft = rng.integers(-4, 5, (g, V)).astype(np.float32) * 0.5
    uni = rng.random(g + 1, dtype=np.float32)
    off = np.array([0, g], np.int32)
    q = oracle.compress(draft, V, T, k)
    tok, _, _ = oracle.sample_draft(q, rng.random(g, dtype=np.float32))
    v = oracle.verify(tgt, V, T, off, tok, q, uni, renorm=renorm)
    r = oracle.sample_residual(tgt, V, T, off, v.n_accept, v.tgt_lse, q, uni, renorm=renorm)
    if v.margin.min() < 1e-9 or r.cdf_margin.min() < 1e-9 or (r.flags[0] & oracle.FLAG_RESIDUAL_EMPTY):
        pytest.skip("knife-edge draw")
    j, pick, R = _brute_round(draft, tgt, T, k, list(tok), [float(x) for x in uni[:g]], float(uni[g]), renorm)
    assert v.n_accept[0] == j
    assert r.out_tok[0] == pick
    np.testing.assert_allclose(r.resid_mass[0], R, rtol=1e-10)


# ---------------------------------------------------------------- edge cases of the layout

def test_ragged_offsets_and_empty_sequences():
    rng = np.random.default_rng(13)
    V = 50
    g = np.array([0, 3, 0, 1], np.int32)
    off = W.seq_offsets(g)
    N, B = 4, 4
    tgt = rng.standard_normal((N + B, V)).astype(np.float32)
    draft = rng.standard_normal((N, V)).astype(np.float32)
    uni = rng.random(N + B, dtype=np.float32)
    q = oracle.compress(draft, V, 1.0, 10)
    tok, _, _ = oracle.sample_draft(q, rng.random(N, dtype=np.float32))
    v = oracle.verify(tgt, V, 1.0, off, tok, q, uni)
    r = oracle.sample_residual(tgt, V, 1.0, off, v.n_accept, v.tgt_lse, q, uni)
    assert v.n_accept[0] == 0 and v.n_accept[2] == 0
    for b in (0, 2):                                                # gamma = 0: bonus token straight from P
        row = off[b] + b
        cdf = np.cumsum(_softmax64(tgt[row], 1.0))
        assert r.out_tok[b] == np.searchsorted(cdf, np.float64(uni[row]) * cdf[-1], side="right")
        assert abs(r.resid_mass[b] - 1.0) < 1e-12
    np.testing.assert_allclose(v.tgt_lse, scipy.special.logsumexp(tgt.astype(np.float64), axis=1), rtol=1e-13)


def test_token_outside_support_is_accepted_and_flagged():
    rng = np.random.default_rng(14)
    V = 30
    off = np.array([0, 2], np.int32)
    tgt = rng.standard_normal((3, V)).astype(np.float32)
    draft = rng.standard_normal((2, V)).astype(np.float32)
    q = oracle.compress(draft, V, 1.0, 5)
    outside = int(np.setdiff1d(np.arange(V), q.idx[0])[0])
    tok = np.array([outside, q.idx[1, 0]], np.int32)
    uni = np.array([0.999, 0.0, 0.5], np.float32)
    v = oracle.verify(tgt, V, 1.0, off, tok, q, uni)
    assert v.n_accept[0] == 2 and v.flags[0] & oracle.FLAG_TOKEN_NOT_IN_SUPPORT
    assert v.q_tok[0] == 0.0


def test_residual_empty_falls_back_to_target():
    V = 6
    z = np.array([[0.0, 1.0, 2.0, -1.0, 0.5, 0.25]], np.float32)
    tgt = np.concatenate([z, z])
    off = np.array([0, 1], np.int32)
    q = oracle.compress(z, V, 1.0, V)
    uni = np.array([0.3, 0.6], np.float32)
    n_acc = np.array([0], np.int32)                                  # force "rejected at 0" with P == Q
    lse = scipy.special.logsumexp(tgt.astype(np.float64), axis=1)
    r = oracle.sample_residual(tgt, V, 1.0, off, n_acc, lse, q, uni)
    assert r.flags[0] & oracle.FLAG_RESIDUAL_EMPTY and r.resid_mass[0] == 0.0
    cdf = np.cumsum(_softmax64(z[0], 1.0))
    assert r.out_tok[0] == np.searchsorted(cdf, np.float64(uni[1]) * cdf[-1], side="right")


def test_sample_draft_is_inverse_cdf_over_slots():
    rng = np.random.default_rng(15)
    z = (rng.standard_normal((200, 40)) * 2).astype(np.float32)
    q = oracle.compress(z, 40, 1.0, 9)
    u = rng.random(200, dtype=np.float32)
    tok, slot, _ = oracle.sample_draft(q, u)
    for r in range(200):
        cdf = np.cumsum(q.prob[r])
        s = int(np.searchsorted(cdf, np.float64(u[r]) * cdf[-1], side="right"))
        assert slot[r] == s and tok[r] == q.idx[r, s]
    # and statistically: slot frequencies follow prob/mass for a repeated row
    zz = np.tile(z[:1], (100_000, 1))
    qq = oracle.compress(zz, 40, 1.0, 9)
    _, sl, _ = oracle.sample_draft(qq, rng.random(100_000, dtype=np.float32))
    exp = qq.prob[0] / qq.mass[0] * 100_000
    assert scipy.stats.chisquare(np.bincount(sl, minlength=9), exp).pvalue > 1e-3


def test_acceptance_is_strict_at_the_boundary():
    """u < min(1, p/q) with equality rejected: V = 1 makes p = 1 exactly, the scalar q makes p/q = 1/2 exactly."""
    tgt = np.zeros((6, 1), np.float32)                       # three sequences, gamma = 1 each
    off = np.array([0, 1, 2, 3], np.int32)
    tok = np.zeros(3, np.int32)
    below = np.nextafter(np.float32(0.5), np.float32(0.0))
    uni = np.array([0.5, 0.0, below, 0.0, np.nextafter(np.float32(0.5), np.float32(1.0)), 0.0], np.float32)
    v = oracle.verify(tgt, 1, 1.0, off, tok, None, uni, q_scalar=np.array([2.0, 2.0, 2.0]))
    assert list(v.p_tok) == [1.0, 1.0, 1.0]
    assert list(v.n_accept) == [0, 1, 0]                     # u == ratio rejects, one ulp below accepts
    assert v.margin[0] == 0.0
