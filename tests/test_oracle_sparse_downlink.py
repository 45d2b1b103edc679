"""Pins of the oracle's paper-literal downlink (Section 3.3: the Top-K record of the target
distribution at the rejected position is sent, Eq. 4, and the edge resamples locally from
norm(max(0, P_j - Q_j)) with its dense Q_j).  CPU only; every check compares the oracle with
something that is not the oracle: a dense numpy implementation written here, a closed form, or
brute force over slots."""
import numpy as np
import pytest
import scipy.special

import oracle
from paper_2603_19133_amd import workloads as W


def _softmax64(z, T):
    return scipy.special.softmax(np.asarray(z, np.float64) / T, axis=-1)


def _case(seed, B=5, V=300, gammas=(3, 0, 4, 1, 2), T=0.9, dtype="f32"):
    rng = np.random.default_rng(seed)
    gam = np.array(gammas[:B], np.int32)
    seq_off = np.concatenate([[0], np.cumsum(gam)]).astype(np.int32)
    N = int(seq_off[-1])
    tgt = (rng.standard_normal((N + B, V)) * 3).astype(np.float32)
    draft = np.empty((max(N, 1), V), np.float32)
    for b in range(B):
        for t in range(gam[b]):
            draft[seq_off[b] + t] = tgt[seq_off[b] + b + t] + rng.standard_normal(V).astype(np.float32)
    if dtype == "bf16":
        tgt_s, draft_s = W.to_bf16_bits(tgt), W.to_bf16_bits(draft)
        tgt, draft = W.bf16_bits_to_f32(tgt_s), W.bf16_bits_to_f32(draft_s)
    else:
        tgt_s, draft_s = tgt, draft
    n_accept = np.array([rng.integers(0, g + 1) for g in gam], np.int32)
    n_accept[0] = gam[0]                      # one bonus position for sure
    uniforms = rng.random(N + B, dtype=np.float32)
    return dict(B=B, V=V, T=T, seq_off=seq_off, gam=gam, tgt=tgt, draft=draft, tgt_s=tgt_s, draft_s=draft_s,
                n_accept=n_accept, uniforms=uniforms)


def _dense_residual(c, b):
    """max(0, P_j - Q_j) over the whole vocabulary, written independently of the oracle."""
    j = int(c["n_accept"][b])
    P = _softmax64(c["tgt"][c["seq_off"][b] + b + j], c["T"])
    if j == c["gam"][b]:
        return P, P, None
    Q = _softmax64(c["draft"][c["seq_off"][b] + j], c["T"])
    return np.maximum(P - Q, 0.0), P, Q


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_record_is_the_topk_of_the_rejected_target_row(dtype):
    c = _case(1, dtype=dtype)
    k = 17
    rec = oracle.compress_rejected(c["tgt_s"], c["V"], c["T"], c["seq_off"], c["n_accept"], k)
    for b in range(c["B"]):
        row = c["tgt"][c["seq_off"][b] + b + c["n_accept"][b]]
        order = np.lexsort((np.arange(c["V"]), -row.astype(np.float64)))[:k]
        assert list(rec.idx[b]) == list(order)
        np.testing.assert_allclose(rec.prob[b], _softmax64(row, c["T"])[order], rtol=1e-12)


@pytest.mark.parametrize("renorm", [0, 1])
def test_full_record_gives_the_exact_residual(renorm):
    """K = V: the record is the whole target distribution, so the weights are max(0, P - Q) itself and
    the residual mass is the closed form 1 - sum min(P, Q)."""
    c = _case(2)
    V = c["V"]
    rec = oracle.compress_rejected(c["tgt_s"], V, c["T"], c["seq_off"], c["n_accept"], V)
    out = oracle.resample_sparse(c["draft_s"], V, c["T"], c["seq_off"], c["n_accept"], rec, c["uniforms"], renorm)
    for b in range(c["B"]):
        r, P, Q = _dense_residual(c, b)
        dense_by_slot = r[rec.idx[b]]
        np.testing.assert_allclose(out.weights[b], dense_by_slot, rtol=1e-9, atol=1e-15)
        R = 1.0 - np.minimum(P, Q).sum() if Q is not None else 1.0
        np.testing.assert_allclose(out.resid_mass[b], R, rtol=1e-9)
        assert out.flags[b] == 0


def test_token_is_the_inverse_cdf_over_slots():
    c = _case(3)
    k = 40
    rec = oracle.compress_rejected(c["tgt_s"], c["V"], c["T"], c["seq_off"], c["n_accept"], k)
    out = oracle.resample_sparse(c["draft_s"], c["V"], c["T"], c["seq_off"], c["n_accept"], rec, c["uniforms"], 0)
    for b in range(c["B"]):
        r, P, Q = _dense_residual(c, b)
        w = [float(r[x]) for x in rec.idx[b]]          # renorm 0: the record's values are P itself
        target = float(c["uniforms"][c["seq_off"][b] + b + c["gam"][b]]) * sum(w)
        cum, pick = 0.0, None
        for s, ws in enumerate(w):                      # brute force, slot order
            cum += ws
            if cum > target:
                pick = s
                break
        assert pick is not None and out.out_tok[b] == rec.idx[b][pick]


def test_bonus_position_draws_from_the_record_itself():
    c = _case(4)
    k = 25
    rec = oracle.compress_rejected(c["tgt_s"], c["V"], c["T"], c["seq_off"], c["n_accept"], k)
    for renorm in (0, 1):
        out = oracle.resample_sparse(c["draft_s"], c["V"], c["T"], c["seq_off"], c["n_accept"], rec, c["uniforms"], renorm)
        b = 0                                           # n_accept[0] = gamma_0
        expect = rec.prob[b] / rec.mass[b] if renorm else rec.prob[b]
        np.testing.assert_allclose(out.weights[b], expect, rtol=1e-14)
        np.testing.assert_allclose(out.resid_mass[b], 1.0 if renorm else rec.mass[b], rtol=1e-12)


def test_truncation_bias_has_its_closed_form_and_vanishes_with_k():
    """renorm 0: the sparse residual is the exact one restricted to the record, so the total-variation
    distance between the two normalised distributions is 1 - R_K / R; it falls with K and is 0 at K = V."""
    c = _case(5, V=2000, gammas=(4, 4, 4, 4, 4))
    c["n_accept"][:] = [1, 2, 0, 3, 2]                   # all at rejected positions
    V = c["V"]
    last = None
    for k in (10, 100, 1000, V):
        rec = oracle.compress_rejected(c["tgt_s"], V, c["T"], c["seq_off"], c["n_accept"], k)
        out = oracle.resample_sparse(c["draft_s"], V, c["T"], c["seq_off"], c["n_accept"], rec, c["uniforms"], 0)
        tvs = []
        for b in range(c["B"]):
            r, _, _ = _dense_residual(c, b)
            exact = r / r.sum()
            sparse = np.zeros(V)
            sparse[rec.idx[b][: rec.count[b]]] = out.weights[b][: rec.count[b]]
            sparse /= sparse.sum()
            tv = 0.5 * np.abs(exact - sparse).sum()
            np.testing.assert_allclose(tv, 1.0 - out.resid_mass[b] / r.sum(), atol=1e-12)
            tvs.append(tv)
        tvs = np.array(tvs)
        if last is not None:
            assert (tvs <= last + 1e-12).all()
        last = tvs
    assert (last < 1e-12).all()


def test_empty_residual_falls_back_to_the_record():
    """Draft == target and K = V: nothing of P exceeds Q; the draw comes from the record and is flagged."""
    c = _case(6)
    for b in range(c["B"]):
        for t in range(c["gam"][b]):
            c["draft_s"][c["seq_off"][b] + t] = c["tgt_s"][c["seq_off"][b] + b + t]
    c["n_accept"][:] = np.minimum(c["n_accept"], np.maximum(c["gam"] - 1, 0))
    V = c["V"]
    rec = oracle.compress_rejected(c["tgt_s"], V, c["T"], c["seq_off"], c["n_accept"], V)
    out = oracle.resample_sparse(c["draft_s"], V, c["T"], c["seq_off"], c["n_accept"], rec, c["uniforms"], 0)
    for b in range(c["B"]):
        if c["n_accept"][b] < c["gam"][b]:
            assert out.flags[b] & oracle.FLAG_RESIDUAL_EMPTY and out.resid_mass[b] == 0.0
            np.testing.assert_allclose(out.weights[b], rec.prob[b], rtol=1e-14)
