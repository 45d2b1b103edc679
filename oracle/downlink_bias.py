"""Truncation bias of the Top-K downlink record (Section 3.3, Eq. 4), computed with the CPU oracle only.

For synthetic rounds of the workloads, the total-variation distance between the exact residual distribution
norm(max(0, P_j - Q_j)) and the one the edge can form from the K-entry record of P_j, as a function of K, with
the record's values used as sent (renorm 0) and renormalised by their mass (renorm 1).  Test infrastructure:
run as ``python -m oracle.downlink_bias``; prints a table (the figures quoted in the design doc)."""
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


def main() -> int:
    for name, B in (("cfg3", 8), ("cfg4", 4), ("cfg5", 8)):
        w = W.WORKLOADS[name]
        print(f"{name}: V={w.V} T={w.T} ({B} sequences, one rejected position each)")
        print("      K   kept mass   TV renorm=0   TV renorm=1")
        for k, m, t0, t1 in tv_table(name, B):
            print(f"  {k:5d}   {m:9.4f}   {t0:11.4f}   {t1:11.4f}")
    return 0


if __name__ == "__main__":
    sys.exit(main())
