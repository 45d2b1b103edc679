"""GPU parity of the wire messages (Section 3.3: uplink of the drafted tokens' own probabilities, downlink
of the Eq. 4 record) through the C ABI against the byte-exact oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_19133_amd import workloads as W

pytestmark = pytest.mark.gpu

FORMATS = [oracle.WIRE_FP32, oracle.WIRE_FP16, oracle.WIRE_BF16]


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


def _batch(seed, B, k, gmax=16, tiny=False):
    """A ragged batch of records as the verifier holds them: fp32 probabilities in descending order per row
    (some rows reaching down into fp16's subnormal range), ids without repeats, counts 0..k."""
    rng = np.random.default_rng(seed)
    g = rng.integers(0, gmax + 1, B)
    seq_off = np.concatenate([[0], np.cumsum(g)]).astype(np.int32)
    n_accept = np.array([rng.integers(0, gi + 1) for gi in g], np.int32)
    count = rng.integers(0, k + 1, B).astype(np.int32)
    count[rng.random(B) < 0.2] = k
    idx = np.full((B, k), -1, np.int32)
    prob = np.zeros((B, k), np.float32)
    for b in range(B):
        c = count[b]
        idx[b, :c] = rng.choice(152064, c, replace=False)
        lo = -30 if (tiny or b % 5 == 0) else -14
        prob[b, :c] = np.sort(np.exp2(rng.uniform(lo, -1, c)))[::-1].astype(np.float32)
    token = rng.integers(0, 152064, B).astype(np.int32)
    return seq_off, n_accept, token, idx, prob, count


def _rec(ps, gpu, idx, prob, count):
    B, k = idx.shape
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(gpu)
    return ps.Compressed(d(idx), d(prob), d(count), torch.zeros(B, device=gpu), torch.zeros(B, device=gpu), k)


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("B,k", [(1, 10), (37, 19), (300, 257), (512, 2048)])
def test_pack_downlink_bytes(gpu, ps, fmt, B, k):
    _announce("pack_downlink", fmt, B, k)
    seq_off, n_accept, token, idx, prob, count = _batch(100 + B, B, k)
    want, n = oracle.pack_downlink(seq_off, n_accept, token, idx, prob, count, fmt)
    d = lambda a: torch.from_numpy(a).to(gpu)
    cap = ps.downlink_bytes_max(B, k, fmt)
    wire = torch.full((cap,), 0xEE, dtype=torch.uint8, device=gpu)
    wire, nbytes, status = ps.pack_downlink(d(seq_off), d(n_accept), d(token), _rec(ps, gpu, idx, prob, count), fmt, wire=wire)
    torch.cuda.synchronize()
    assert int(nbytes.item()) == n and int(status.item()) == 0
    got = wire.cpu().numpy()
    assert np.array_equal(got[:n], want)
    assert np.all(got[n:] == 0xEE)                      # nothing behind the message is touched


@pytest.mark.parametrize("fmt", FORMATS)
def test_pack_downlink_too_small_a_buffer_and_tokens_only(gpu, ps, fmt):
    _announce("pack_downlink small", fmt)
    B, k = 21, 33
    seq_off, n_accept, token, idx, prob, count = _batch(7, B, k)
    want, n = oracle.pack_downlink(seq_off, n_accept, token, idx, prob, count, fmt)
    d = lambda a: torch.from_numpy(a).to(gpu)
    small = torch.full((n - 4,), 0xEE, dtype=torch.uint8, device=gpu)
    _, nbytes, status = ps.pack_downlink(d(seq_off), d(n_accept), d(token), _rec(ps, gpu, idx, prob, count), fmt, wire=small)
    torch.cuda.synchronize()
    assert int(nbytes.item()) == n and int(status.item()) == ps.WIRE_TRUNCATED
    assert bool((small == 0xEE).all())
    exact = torch.full((n,), 0xEE, dtype=torch.uint8, device=gpu)
    _, nbytes, status = ps.pack_downlink(d(seq_off), d(n_accept), d(token), _rec(ps, gpu, idx, prob, count), fmt, wire=exact)
    assert int(status.item()) == 0 and np.array_equal(exact.cpu().numpy(), want)
    # tokens only; and without tokens at all
    want, n = oracle.pack_downlink(seq_off, n_accept, token, None, None, None, fmt)
    wire, nbytes, status = ps.pack_downlink(d(seq_off), d(n_accept), d(token), None, fmt)
    assert int(nbytes.item()) == n == 8 + 8 * B and np.array_equal(wire.cpu().numpy()[:n], want)
    want, n = oracle.pack_downlink(seq_off, n_accept, None, idx, prob, count, fmt)
    wire, nbytes, status = ps.pack_downlink(d(seq_off), d(n_accept), None, _rec(ps, gpu, idx, prob, count), fmt)
    assert int(nbytes.item()) == n and np.array_equal(wire.cpu().numpy()[:n], want)
    # an empty batch is the header alone
    want, n = oracle.pack_downlink(np.zeros(1, np.int32), np.zeros(0, np.int32), None, None, None, None, fmt)
    wire, nbytes, status = ps.pack_downlink(torch.zeros(1, dtype=torch.int32, device=gpu),
                                            torch.zeros(0, dtype=torch.int32, device=gpu), None, None, fmt)
    assert int(nbytes.item()) == n == 8 and np.array_equal(wire.cpu().numpy()[:8], want)


def _compare_unpacked(pu, g, o, k):
    assert int(g.status.item()) == o.status
    if o.status & (oracle.WIRE_BAD_HEADER | oracle.WIRE_BAD_BATCH | oracle.WIRE_TRUNCATED):
        return
    assert np.array_equal(pu.n(g.n_accept), o.n_accept) and np.array_equal(pu.n(g.token), o.token)
    assert np.array_equal(pu.n(g.rec.count), o.count) and np.array_equal(pu.n(g.rec.idx), o.idx)
    assert np.array_equal(pu.n(g.rec.prob).astype(np.float64), o.prob)       # widening is exact
    pu.assert_close(pu.n(g.rec.mass), o.mass, 1e-6, "mass of the received record", atol=1e-38)


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("B,k", [(1, 10), (37, 19), (300, 257), (512, 2048)])
def test_unpack_downlink(gpu, ps, pu, fmt, B, k):
    _announce("unpack_downlink", fmt, B, k)
    seq_off, n_accept, token, idx, prob, count = _batch(200 + B, B, k)
    wire, n = oracle.pack_downlink(seq_off, n_accept, token, idx, prob, count, fmt)
    dw = torch.from_numpy(wire).to(gpu)
    _compare_unpacked(pu, ps.unpack_downlink(dw, n, B, k), oracle.unpack_downlink(wire, B, k), k)
    if k > 4:      # a receiver with fewer slots keeps the front of every record
        k2 = k // 2
        o = oracle.unpack_downlink(wire, B, k2)
        _compare_unpacked(pu, ps.unpack_downlink(dw, n, B, k2), o, k2)
        assert o.status == (oracle.WIRE_CLAMPED if (np.where(n_accept < np.diff(seq_off), count, 0) > k2).any() else 0)


def test_unpack_downlink_statuses(gpu, ps, pu):
    _announce("unpack_downlink statuses")
    B, k = 9, 12
    seq_off, n_accept, token, idx, prob, count = _batch(5, B, k)
    wire, n = oracle.pack_downlink(seq_off, n_accept, token, idx, prob, count, oracle.WIRE_FP16)
    cases = {"short": (wire[:n - 4], B), "entries cut": (wire[:16], B), "no header": (wire[:4], B), "batch": (wire, B + 1)}
    for name, byte, val in (("magic", 0, wire[0] ^ 1), ("version", 2, 9), ("format", 3, 3)):
        bad = wire.copy()
        bad[byte] = val
        cases[name] = (bad, B)
    up, _ = oracle.pack_uplink(np.array([0, 2]), np.array([5, 6]), np.array([0.5, 0.25], np.float32), oracle.WIRE_FP32)
    cases["an uplink message"] = (up, 1)
    for name, (w, Bn) in cases.items():
        o = oracle.unpack_downlink(w, Bn, k)
        assert o.status != 0, name
        buf = torch.zeros(max(len(w), 4), dtype=torch.uint8, device=gpu)
        buf[:len(w)] = torch.from_numpy(w).to(gpu)
        assert int(ps.unpack_downlink(buf, len(w), Bn, k).status.item()) == o.status, name
    # nothing but the status is written on such a message
    out = ps.Downlink(torch.full((B,), -5, dtype=torch.int32, device=gpu), torch.full((B,), -5, dtype=torch.int32, device=gpu),
                      ps.Compressed(torch.full((B, k), -5, dtype=torch.int32, device=gpu), torch.full((B, k), -5.0, device=gpu), torch.full((B,), -5, dtype=torch.int32, device=gpu),
                                    torch.full((B,), -5.0, device=gpu), torch.zeros(B, device=gpu), k),
                      torch.zeros(1, dtype=torch.int32, device=gpu))
    short = torch.from_numpy(wire[:n - 4].copy()).to(gpu)
    ps._check(ps.lib.picospec_unpack_downlink(short.data_ptr(), n - 4, B, k, out.n_accept.data_ptr(), out.token.data_ptr(),
                                              out.rec.idx.data_ptr(), out.rec.prob.data_ptr(), out.rec.count.data_ptr(),
                                              out.rec.mass.data_ptr(), out.status.data_ptr(), None))
    torch.cuda.synchronize()
    assert int(out.status.item()) == ps.WIRE_TRUNCATED
    assert bool((out.rec.idx == -5).all()) and bool((out.n_accept == -5).all()) and bool((out.rec.mass == -5.0).all())


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("B,gmax", [(1, 6), (29, 16), (512, 16), (1000, 3)])
def test_uplink_pack_and_unpack(gpu, ps, pu, fmt, B, gmax):
    _announce("uplink", fmt, B, gmax)
    rng = np.random.default_rng(B + fmt)
    g = rng.integers(0, gmax + 1, B)
    seq_off = np.concatenate([[0], np.cumsum(g)]).astype(np.int32)
    N = int(seq_off[-1])
    tok = rng.integers(0, 152064, N).astype(np.int32)
    q = np.exp2(rng.uniform(-28, 0, N)).astype(np.float32)
    want, n = oracle.pack_uplink(seq_off, tok, q, fmt)
    d = lambda a: torch.from_numpy(a).to(gpu)
    assert ps.uplink_bytes(B, N, fmt) == n
    wire = torch.full((n + 16,), 0xEE, dtype=torch.uint8, device=gpu)
    _, nbytes = ps.pack_uplink(d(seq_off), N, d(tok), d(q), fmt, wire=wire)
    torch.cuda.synchronize()
    got = wire.cpu().numpy()
    assert int(nbytes.item()) == n and np.array_equal(got[:n], want) and np.all(got[n:] == 0xEE)
    for n_max in sorted({N, N + 5, N // 2, 0}):
        o = oracle.unpack_uplink(want, B, n_max)
        so, t, qq, st = ps.unpack_uplink(d(want), n, B, n_max)
        torch.cuda.synchronize()
        assert int(st.item()) == o.status
        assert np.array_equal(pu.n(so), o.seq_off)
        kept = int(o.seq_off[-1])
        assert np.array_equal(pu.n(t)[:kept], o.draft_tok[:kept])
        assert np.array_equal(pu.n(qq)[:kept].astype(np.float64), o.q_scalar[:kept])
    for name, w, Bn in (("short", want[:n - 4], B), ("batch", want, B + 1), ("magic", np.concatenate([[0x50], want[1:]]).astype(np.uint8), B)):
        o = oracle.unpack_uplink(np.ascontiguousarray(w), Bn, N)
        buf = torch.zeros(max(len(w), 4), dtype=torch.uint8, device=gpu)
        buf[:len(w)] = torch.from_numpy(np.ascontiguousarray(w)).to(gpu)
        *_, st = ps.unpack_uplink(buf, len(w), Bn, N)
        assert int(st.item()) == o.status != 0, name


@pytest.mark.parametrize("cfg,k", [("cfg1", 64), ("cfg3", 1024)])
def test_round_over_the_wire(gpu, ps, pu, cfg, k):
    """One round as the paper ships it, both messages through the library: the edge's scalars go up, the
    verifier's records come down, the edge resamples.  With fp32 probabilities the wire changes nothing;
    with fp16 the received record equals the oracle's reading of the oracle's bytes."""
    _announce("round over the wire", cfg, k)
    w = W.WORKLOADS[cfg]
    r = W.build_round(w, 0)
    draft, tgt = pu.to_device(r.draft_logits, gpu), pu.to_device(r.tgt_logits, gpu)
    seq_off = torch.from_numpy(r.seq_off).to(gpu)
    uni, duni = torch.from_numpy(r.uniforms).to(gpu), torch.from_numpy(r.draft_uniforms).to(gpu)
    q = ps.compress(draft, w.V, w.T, min(w.V, 4096))
    tok, q_scalar = ps.sample_draft(q, duni)
    # uplink, fp32: what the verifier unpacks is what the edge held
    up, nb = ps.pack_uplink(seq_off, r.N, tok, q_scalar, ps.WIRE_FP32)
    so2, tok2, q2, st = ps.unpack_uplink(up, int(nb.item()), r.B, r.N)
    assert int(st.item()) == 0 and torch.equal(so2, seq_off) and torch.equal(tok2, tok) and torch.equal(q2, q_scalar)
    ver = ps.verify(tgt, w.V, w.T, so2, r.N, tok2, None, uni, q_scalar=q2)
    rec = ps.compress_rejected(tgt, w.V, w.T, seq_off, r.N, ver.n_accept, k)
    dmax, dsum, _ = ps.row_stats(draft, w.V, w.T)
    direct = ps.resample_sparse(draft, w.V, w.T, seq_off, r.N, ver.n_accept, dmax, dsum, rec, uni, 0)
    # downlink, fp32: identical tokens; sequences without a rejection carry no record
    down, nb, st = ps.pack_downlink(seq_off, ver.n_accept, None, rec, ps.WIRE_FP32)
    got = ps.unpack_downlink(down, int(nb.item()), r.B, k)
    assert int(st.item()) == 0 and int(got.status.item()) == 0 and torch.equal(got.n_accept, ver.n_accept)
    rejected = ver.n_accept < (seq_off[1:] - seq_off[:-1])
    assert torch.equal(got.rec.count, torch.where(rejected, rec.count, torch.zeros_like(rec.count)))
    via = ps.resample_sparse(draft, w.V, w.T, seq_off, r.N, got.n_accept, dmax, dsum, got.rec, uni, 0)
    torch.cuda.synchronize()
    rj = rejected.cpu().numpy()
    assert rj.any()
    assert np.array_equal(pu.n(via.out_tok)[rj], pu.n(direct.out_tok)[rj])
    assert np.array_equal(pu.n(via.resid_mass)[rj], pu.n(direct.resid_mass)[rj])
    assert np.all(pu.n(via.out_tok)[~rj] == -1)          # nothing came down for them: the edge has no record to draw from


@pytest.mark.parametrize("fmt", [oracle.WIRE_FP16, oracle.WIRE_BF16])
@pytest.mark.parametrize("cfg,k", [("cfg1", 64), ("cfg2", 256)])
def test_local_resampling_from_a_quantised_downlink(gpu, ps, pu, fmt, cfg, k):
    """The edge's draw from a record that crossed the wire with 16-bit probabilities: oracle chain (record,
    bytes, received record, local resampling) against the library's on the same record and uniforms."""
    _announce("quantised downlink", fmt, cfg, k)
    w = W.WORKLOADS[cfg]
    r = W.build_round(w, 0)
    rng = np.random.default_rng(17)
    g = np.diff(r.seq_off)
    na = np.array([rng.integers(0, gi) if gi > 0 else 0 for gi in g], np.int32)      # every sequence rejects somewhere
    orec = oracle.compress_rejected(r.tgt_logits, w.V, w.T, r.seq_off, na, k)
    prob32 = orec.prob.astype(np.float32)
    wire, n = oracle.pack_downlink(r.seq_off, na, None, orec.idx, prob32, orec.count, fmt)
    od = oracle.unpack_downlink(wire, r.B, k)
    received = oracle.Compressed(od.idx, od.prob, od.count, od.mass, None, None, k)
    ores = oracle.resample_sparse(r.draft_logits, w.V, w.T, r.seq_off, od.n_accept, received, r.uniforms, 0)

    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(gpu)
    draft = pu.to_device(r.draft_logits, gpu)
    seq_off, uni = d(r.seq_off), d(r.uniforms)
    gw, nb, st = ps.pack_downlink(seq_off, d(na), None, _rec(ps, gpu, orec.idx, prob32, orec.count), fmt)
    assert int(nb.item()) == n and int(st.item()) == 0 and np.array_equal(gw.cpu().numpy()[:n], wire)
    got = ps.unpack_downlink(gw, n, r.B, k)
    _compare_unpacked(pu, got, od, k)
    dmax, dsum, _ = ps.row_stats(draft, w.V, w.T)
    gres = ps.resample_sparse(draft, w.V, w.T, seq_off, r.N, got.n_accept, dmax, dsum, got.rec, uni, 0)
    torch.cuda.synchronize()
    assert (pu.n(gres.flags).astype(np.uint32) == ores.flags).all()
    pu.assert_close(pu.n(gres.resid_mass), ores.resid_mass, pu.RTOL, "resid_mass", atol=1e-30)
    same = pu.n(gres.out_tok) == ores.out_tok
    assert np.all(same | (ores.cdf_margin < pu.CDF_MARGIN))
