"""Truncation bias of the Top-K downlink record (Section 3.3, Eq. 4), computed with the CPU oracle only.

For synthetic rounds of the workloads, the total-variation distance between the exact residual distribution
norm(max(0, P_j - Q_j)) and the one the edge can form from the K-entry record of P_j, as a function of K, with
the record's values used as sent (renorm 0) and renormalised by their mass (renorm 1); and what 16-bit
probabilities on the wire cost on top: the total variation between the edge's draw from the received record and
from the fp32 record, and the change of the acceptance probabilities when the uplinked q_i are quantised.
Test infrastructure: run as ``python -m oracle.downlink_bias``; prints tables of the sparse downlink's bias."""
from __future__ import annotations

import sys

import numpy as np
import scipy.special

import oracle
from paper_2603_19133_amd import workloads as W


def tv_table(name: str, B: int, ks=(10, 64, 256, 1024, 4096)):
    w = W.WORKLOADS[name].scaled(B=B)
    r = W.build_round(w, 0)
    rng = np.random.default_rng(7)
    gam = np.diff(r.seq_off)
    na = np.array([rng.integers(0, g) if g > 0 else 0 for g in gam], np.int32)   # a rejected position everywhere
    rows = []
    f32 = lambda a: W.bf16_bits_to_f32(a) if a.dtype == np.uint16 else a
    for k in ks:
        rec = oracle.compress_rejected(r.tgt_logits, w.V, w.T, r.seq_off, na, k)
        out = []
        for renorm in (0, 1):
            res = oracle.resample_sparse(r.draft_logits, w.V, w.T, r.seq_off, na, rec, r.uniforms, renorm)
            tvs = []
            for b in range(r.B):
                if gam[b] == 0:
                    continue
                P = scipy.special.softmax(f32(r.tgt_logits[r.seq_off[b] + b + na[b]]).astype(np.float64) / w.T)
                Q = scipy.special.softmax(f32(r.draft_logits[r.seq_off[b] + na[b]]).astype(np.float64) / w.T)
                exact = np.maximum(P - Q, 0.0)
                exact /= exact.sum()
                sparse = np.zeros(w.V)
                c = rec.count[b]
                sparse[rec.idx[b][:c]] = res.weights[b][:c]
                sparse /= sparse.sum()
                tvs.append(0.5 * np.abs(exact - sparse).sum())
            out.append(float(np.mean(tvs)))
        rows.append((k, float(rec.mass.mean()), out[0], out[1]))
    return rows


def quantisation_table(name: str, B: int, ks=(10, 64, 1024, 4096)):
    """Per K and wire format: bytes of one record on the downlink; mean total variation between the edge's draw
    from the received record and from the fp32 record.  Then, per format, the uplink: mean and largest change of
    the acceptance probability min(1, p_i / q_i) and the number of sequences whose accepted length changes."""
    w = W.WORKLOADS[name].scaled(B=B)
    r = W.build_round(w, 0)
    rng = np.random.default_rng(7)
    gam = np.diff(r.seq_off)
    na = np.array([rng.integers(0, g) if g > 0 else 0 for g in gam], np.int32)
    fmts = ((oracle.WIRE_FP32, "fp32"), (oracle.WIRE_FP16, "fp16"), (oracle.WIRE_BF16, "bf16"))
    down = []
    for k in ks:
        rec = oracle.compress_rejected(r.tgt_logits, w.V, w.T, r.seq_off, na, k)
        p32 = rec.prob.astype(np.float32)
        ref = None
        for fmt, label in fmts:
            wire, n = oracle.pack_downlink(r.seq_off, na, None, rec.idx, p32, rec.count, fmt)
            got = oracle.unpack_downlink(wire, r.B, k)
            received = oracle.Compressed(got.idx, got.prob, got.count, got.mass, None, None, k)
            res = oracle.resample_sparse(r.draft_logits, w.V, w.T, r.seq_off, na, received, r.uniforms, 0)
            dist = res.weights / res.weights.sum(axis=1, keepdims=True)
            if ref is None:
                ref = dist
            tv = float(np.mean(0.5 * np.abs(dist - ref).sum(axis=1)))
            down.append((k, label, (n - 8 - 8 * r.B) / r.B, tv))
    qd = oracle.compress(r.draft_logits, w.V, w.T, min(w.V, 4096))
    tok, slot, _ = oracle.sample_draft(qd, r.draft_uniforms)
    q32 = (qd.prob[np.arange(r.N), slot] / qd.mass).astype(np.float32)
    up = []
    base = None
    for fmt, label in fmts:
        wire, n = oracle.pack_uplink(r.seq_off, tok, q32, fmt)
        got = oracle.unpack_uplink(wire, r.B, r.N)
        v = oracle.verify(r.tgt_logits, w.V, w.T, r.seq_off, got.draft_tok, None, r.uniforms, q_scalar=got.q_scalar)
        acc = np.minimum(1.0, v.p_tok / v.q_tok)
        if base is None:
            base = (acc, v.n_accept)
        d = np.abs(acc - base[0])
        up.append((label, n, float(d.mean()), float(d.max()), int((v.n_accept != base[1]).sum())))
    return down, up


def main() -> int:
    for name, B in (("cfg3", 8), ("cfg4", 4), ("cfg5", 8)):
        w = W.WORKLOADS[name]
        print(f"{name}: V={w.V} T={w.T} ({B} sequences, one rejected position each)")
        print("      K   kept mass   TV renorm=0   TV renorm=1")
        for k, m, t0, t1 in tv_table(name, B):
            print(f"  {k:5d}   {m:9.4f}   {t0:11.4f}   {t1:11.4f}")
    for name, B in (("cfg3", 8), ("cfg4", 4), ("cfg5", 8)):
        down, up = quantisation_table(name, B)
        print(f"{name}: probabilities on the wire")
        print("      K  format  bytes/record  TV against the fp32 record")
        for k, label, nbytes, tv in down:
            print(f"  {k:5d}  {label:6s}  {nbytes:12.0f}  {tv:.2e}")
        print("  uplink format  bytes  mean |d accept prob|  max |d accept prob|  sequences with another accepted length")
        for label, n, dm, dx, ch in up:
            print(f"  {label:13s}  {n:5d}  {dm:.2e}  {dx:.2e}  {ch}")
    return 0


if __name__ == "__main__":
    sys.exit(main())
