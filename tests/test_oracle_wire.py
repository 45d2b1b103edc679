"""Pins of the wire-message oracle (paper Section 3.3: uplink of the drafted tokens' own probabilities,
downlink of the Eq. 4 Top-K record, laid out for in-place views) against things other than itself:
hand-written bytes, the paper's payload sizes, numpy's and torch's fp16/bf16 converters, an independent
numpy decoder of the layout, round trips and the error statuses."""
import os
import re

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "wire_small.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or ":" not in line:
            continue
        name, hexs = line.split(":", 1)
        out[name.strip()] = bytes.fromhex(re.sub(r"\s+", "", hexs))
    return out


SMALL = dict(seq_off=np.array([0, 2, 5]), n_accept=np.array([1, 3]), token=np.array([7, 9]),
             idx=np.array([[5, 3, -1], [1, 2, 3]]), prob=np.array([[0.5, 0.25, 0], [0.1, 0.2, 0.3]], np.float32),
             count=np.array([2, 3]))


@pytest.mark.parametrize("fmt,name", [(oracle.WIRE_FP32, "down_fp32"), (oracle.WIRE_FP16, "down_fp16"),
                                      (oracle.WIRE_BF16, "down_bf16")])
def test_downlink_bytes_of_a_hand_written_message(fmt, name):
    want = _golden()[name]
    wire, n = oracle.pack_downlink(SMALL["seq_off"], SMALL["n_accept"], SMALL["token"], SMALL["idx"],
                                   SMALL["prob"], SMALL["count"], fmt)
    assert n == len(want) and wire.tobytes() == want
    d = oracle.unpack_downlink(np.frombuffer(want, np.uint8), 2, 3)
    assert d.status == 0
    assert d.n_accept.tolist() == [1, 3] and d.token.tolist() == [-1, 9] and d.count.tolist() == [2, 0]
    assert d.idx.tolist() == [[5, 3, -1], [-1, -1, -1]]
    assert d.prob.tolist() == [[0.5, 0.25, 0.0], [0.0, 0.0, 0.0]] and d.mass.tolist() == [0.75, 0.0]


def test_uplink_bytes_of_hand_written_messages():
    g = _golden()
    wire, n = oracle.pack_uplink(np.array([0, 2, 3]), np.array([100, 200, 70000]),
                                 np.array([0.5, 0.125, 1.0], np.float32), oracle.WIRE_FP16)
    assert n == 32 and wire.tobytes() == g["up_fp16"]
    wire, n = oracle.pack_uplink(np.array([0, 1]), np.array([5]), np.array([0.75], np.float32), oracle.WIRE_FP32)
    assert n == 20 and wire.tobytes() == g["up_fp32"]
    u = oracle.unpack_uplink(np.frombuffer(g["up_fp16"], np.uint8), 2, 3)
    assert u.status == 0 and u.seq_off.tolist() == [0, 2, 3]
    assert u.draft_tok.tolist() == [100, 200, 70000] and u.q_scalar.tolist() == [0.5, 0.125, 1.0]


def test_payload_sizes_the_paper_states():
    """Section 3.3: a K = 10 record is 80 bytes of entries and the message stays under 100 bytes; six drafted
    tokens with their probabilities are 48 bytes (under 50), and the whole message is with fp16 probabilities."""
    K = 10
    idx = np.arange(K, dtype=np.int32)[None]
    prob = np.full((1, K), 0.05, np.float32)
    _, n = oracle.pack_downlink(np.array([0, 4]), np.array([2]), None, idx, prob, np.array([K]), oracle.WIRE_FP32)
    assert n - 8 - 8 == 80 and n < 100
    _, n32 = oracle.pack_uplink(np.array([0, 6]), np.arange(6), np.full(6, 0.5, np.float32), oracle.WIRE_FP32)
    _, n16 = oracle.pack_uplink(np.array([0, 6]), np.arange(6), np.full(6, 0.5, np.float32), oracle.WIRE_FP16)
    assert n32 - 8 - 4 == 48 and n16 < 50
    assert oracle.record_bytes() == 8


def _probe_values():
    rng = np.random.default_rng(5)
    vals = [np.exp2(rng.uniform(-30, 1, 200000)).astype(np.float32),          # probabilities over 9 decades
            rng.random(100000, dtype=np.float32),
            (rng.standard_normal(50000) * 1e4).astype(np.float32),
            np.array([0.0, -0.0, 1.0, 0.1, 65504.0, 65519.99, 65520.0, 1e6, -1e6, 2.0 ** -24, 2.0 ** -25,
                      1.5 * 2.0 ** -25, 1.5 * 2.0 ** -24, 2.0 ** -14, np.inf, -np.inf, 6.1e-5, 5.96e-8], np.float32)]
    # every tie between neighbouring halfs and bfloat16s in the probability range, and its fp32 neighbours
    h = np.arange(0, 0x3C01, dtype=np.uint16).view(np.float16).astype(np.float64)
    mid = ((h[:-1] + h[1:]) / 2).astype(np.float32)
    vals += [mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(2))]
    b = (np.arange(0x3000, 0x3F81, dtype=np.uint32) << 16).view(np.float32).astype(np.float64)
    midb = ((b[:-1] + b[1:]) / 2).astype(np.float32)
    vals += [midb, np.nextafter(midb, np.float32(0)), np.nextafter(midb, np.float32(2))]
    return np.concatenate(vals)


def test_fp16_rounding_is_numpys():
    v = _probe_values()
    bits, back = oracle.wire_quantise(v, oracle.WIRE_FP16)
    with np.errstate(over="ignore"):
        want = v.astype(np.float16)
    assert np.array_equal(bits, want.view(np.uint16))
    assert np.array_equal(back, want.astype(np.float64))
    g = {0.1: 0x2E66, 65520.0: 0x7C00, 2.0 ** -25: 0, 1.5 * 2.0 ** -25: 1, 1.5 * 2.0 ** -24: 2}
    for x, b in g.items():
        assert oracle.wire_quantise(np.array([x], np.float32), oracle.WIRE_FP16)[0][0] == b


def test_bf16_rounding_is_torchs():
    v = _probe_values()
    bits, back = oracle.wire_quantise(v, oracle.WIRE_BF16)
    want = torch.from_numpy(v).to(torch.bfloat16)
    assert np.array_equal(bits, want.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(back, want.to(torch.float64).numpy())
    assert oracle.wire_quantise(np.array([0.1], np.float32), oracle.WIRE_BF16)[0][0] == 0x3DCD


def _random_batch(seed, B, k, gmax=9):
    rng = np.random.default_rng(seed)
    g = rng.integers(0, gmax + 1, B)
    seq_off = np.concatenate([[0], np.cumsum(g)]).astype(np.int32)
    n_accept = np.array([rng.integers(0, gi + 1) for gi in g], np.int32)
    count = rng.integers(0, k + 1, B).astype(np.int32)
    idx = np.full((B, k), -1, np.int32)
    prob = np.zeros((B, k), np.float32)
    for b in range(B):
        idx[b, :count[b]] = rng.choice(150000, count[b], replace=False)
        p = np.sort(rng.dirichlet(np.full(max(count[b], 1), 0.3)))[::-1][:count[b]]
        prob[b, :count[b]] = (p * 0.97).astype(np.float32)
    token = rng.integers(0, 150000, B).astype(np.int32)
    return seq_off, n_accept, token, idx, prob, count


def _decode_downlink_with_numpy_views(wire: bytes):
    """An independent reader: the arrays as in-place views at the offsets the format defines."""
    buf = np.frombuffer(wire, np.uint8)
    magic, = buf[0:2].view("<u2")
    version, fmt = int(buf[2]), int(buf[3])
    B = int(buf[4:8].view("<u4")[0])
    ent = buf[8:8 + 8 * B].view(np.dtype([("na", "<u2"), ("cnt", "<u2"), ("tok", "<i4")]))
    total = int(ent["cnt"].sum())
    ids = buf[8 + 8 * B: 8 + 8 * B + 4 * total].view("<i4")
    pdt = {0: "<f4", 1: "<f2"}.get(fmt)
    at = 8 + 8 * B + 4 * total
    if pdt:
        probs = buf[at: at + np.dtype(pdt).itemsize * total].view(pdt).astype(np.float64)
    else:
        probs = (buf[at: at + 2 * total].view("<u2").astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return magic, version, fmt, B, ent, ids, probs


@pytest.mark.parametrize("fmt", [oracle.WIRE_FP32, oracle.WIRE_FP16, oracle.WIRE_BF16])
def test_downlink_layout_read_back_by_an_independent_decoder(fmt):
    seq_off, n_accept, token, idx, prob, count = _random_batch(11, 37, 19)
    wire, n = oracle.pack_downlink(seq_off, n_accept, token, idx, prob, count, fmt)
    magic, version, f, B, ent, ids, probs = _decode_downlink_with_numpy_views(wire.tobytes())
    assert (magic, version, f, B) == (0x5350, 1, fmt, 37) and n % 4 == 0
    g = np.diff(seq_off)
    rejected = n_accept < g
    assert np.array_equal(ent["na"], n_accept) and np.array_equal(ent["cnt"], np.where(rejected, count, 0))
    assert np.array_equal(ent["tok"], np.where(np.where(rejected, count, 0) == 0, token, -1))
    want_ids = np.concatenate([idx[b, :count[b]] for b in range(37) if rejected[b]])
    want_p = np.concatenate([prob[b, :count[b]] for b in range(37) if rejected[b]])
    assert np.array_equal(ids, want_ids)
    if fmt == oracle.WIRE_FP32:
        assert np.array_equal(probs, want_p.astype(np.float64))
    elif fmt == oracle.WIRE_FP16:
        assert np.array_equal(probs, want_p.astype(np.float16).astype(np.float64))
    else:
        assert np.array_equal(probs, torch.from_numpy(want_p).to(torch.bfloat16).to(torch.float64).numpy())


@pytest.mark.parametrize("fmt,rel", [(oracle.WIRE_FP32, 0.0), (oracle.WIRE_FP16, 2.0 ** -11), (oracle.WIRE_BF16, 2.0 ** -8)])
def test_downlink_round_trip(fmt, rel):
    B, k = 41, 23
    seq_off, n_accept, token, idx, prob, count = _random_batch(3, B, k)
    wire, _ = oracle.pack_downlink(seq_off, n_accept, token, idx, prob, count, fmt)
    d = oracle.unpack_downlink(wire, B, k)
    assert d.status == 0
    rejected = n_accept < np.diff(seq_off)
    assert np.array_equal(d.n_accept, n_accept)
    assert np.array_equal(d.count, np.where(rejected, count, 0))
    for b in range(B):
        c = d.count[b]
        assert np.array_equal(d.idx[b, :c], idx[b, :c]) and np.all(d.idx[b, c:] == -1) and np.all(d.prob[b, c:] == 0)
        p = prob[b, :c].astype(np.float64)
        normal = p >= 2.0 ** -14                      # fp16 keeps 11 significant bits only above its smallest normal
        assert np.all(np.abs(d.prob[b, :c] - p)[normal] <= rel * p[normal])
        assert np.all(np.abs(d.prob[b, :c] - p)[~normal] <= (2.0 ** -25 if fmt == oracle.WIRE_FP16 else rel * p[~normal]))
        assert d.mass[b] == pytest.approx(float(np.sum(d.prob[b, :c])), rel=1e-15, abs=0)
        assert d.token[b] == (token[b] if c == 0 else -1)


def test_tokens_only_downlink():
    """The cloud may decide every token itself (dense residual on the verifier): no records, 8 bytes per sequence."""
    seq_off, n_accept, token, *_ = _random_batch(8, 13, 4)
    wire, n = oracle.pack_downlink(seq_off, n_accept, token, None, None, None, oracle.WIRE_FP32)
    assert n == 8 + 8 * 13
    d = oracle.unpack_downlink(wire, 13, 4)
    assert d.status == 0 and np.array_equal(d.token, token) and np.all(d.count == 0) and np.all(d.idx == -1)


@pytest.mark.parametrize("fmt", [oracle.WIRE_FP32, oracle.WIRE_FP16, oracle.WIRE_BF16])
def test_uplink_round_trip_and_layout(fmt):
    rng = np.random.default_rng(21)
    B = 29
    g = rng.integers(0, 17, B)
    seq_off = np.concatenate([[0], np.cumsum(g)]).astype(np.int32)
    N = int(seq_off[-1])
    tok = rng.integers(0, 152064, N).astype(np.int32)
    q = rng.random(N, dtype=np.float32)
    wire, n = oracle.pack_uplink(seq_off, tok, q, fmt)
    w = 4 if fmt == oracle.WIRE_FP32 else 2
    tok_at = 8 + (2 * B + 3) // 4 * 4
    assert n == (tok_at + 4 * N + w * N + 3) // 4 * 4
    buf = wire
    assert np.array_equal(buf[8:8 + 2 * B].view("<u2"), g) and np.array_equal(buf[tok_at:tok_at + 4 * N].view("<i4"), tok)
    u = oracle.unpack_uplink(wire, B, N)
    assert u.status == 0 and np.array_equal(u.seq_off, seq_off) and np.array_equal(u.draft_tok, tok)
    if fmt == oracle.WIRE_FP32:
        assert np.array_equal(u.q_scalar, q.astype(np.float64))
    elif fmt == oracle.WIRE_FP16:
        assert np.array_equal(u.q_scalar, q.astype(np.float16).astype(np.float64))
    else:
        assert np.array_equal(u.q_scalar, torch.from_numpy(q).to(torch.bfloat16).to(torch.float64).numpy())


def test_statuses():
    B, k = 6, 5
    seq_off, n_accept, token, idx, prob, count = _random_batch(2, B, k)
    n_accept[:] = 0
    seq_off = np.arange(0, 2 * B + 1, 2, dtype=np.int32)      # every sequence rejected at once
    count[:] = k
    wire, n = oracle.pack_downlink(seq_off, n_accept, token, idx, prob, count, oracle.WIRE_FP16)
    assert oracle.unpack_downlink(wire, B, k).status == 0
    assert oracle.unpack_downlink(wire[:-4], B, k).status == oracle.WIRE_TRUNCATED
    assert oracle.unpack_downlink(wire[:20], B, k).status == oracle.WIRE_TRUNCATED
    assert oracle.unpack_downlink(wire, B + 1, k).status == oracle.WIRE_BAD_BATCH
    bad = wire.copy(); bad[0] ^= 1
    assert oracle.unpack_downlink(bad, B, k).status == oracle.WIRE_BAD_HEADER
    bad = wire.copy(); bad[2] = 2
    assert oracle.unpack_downlink(bad, B, k).status == oracle.WIRE_BAD_HEADER
    bad = wire.copy(); bad[3] = 3
    assert oracle.unpack_downlink(bad, B, k).status == oracle.WIRE_BAD_HEADER
    d = oracle.unpack_downlink(wire, B, k - 2)                # receiver with fewer slots: the front of each record
    assert d.status == oracle.WIRE_CLAMPED and np.all(d.count == k - 2)
    for b in range(B):
        assert np.array_equal(d.idx[b], idx[b, :k - 2])
    # a buffer too small for the message: nothing written, the size reported
    w2, n2 = oracle.pack_downlink(seq_off, n_accept, token, idx, prob, count, oracle.WIRE_FP16, capacity=n - 1)
    assert w2 is None and n2 == n
    # the uplink's own magic is not the downlink's
    up, _ = oracle.pack_uplink(np.array([0, 1]), np.array([5]), np.array([0.5], np.float32), oracle.WIRE_FP32)
    assert oracle.unpack_downlink(up, 1, 1).status == oracle.WIRE_BAD_HEADER
    assert oracle.unpack_uplink(wire, B, 100).status == oracle.WIRE_BAD_HEADER
    u = oracle.unpack_uplink(up, 1, 0)
    assert u.status == oracle.WIRE_CLAMPED and u.seq_off.tolist() == [0, 0]
