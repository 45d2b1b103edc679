#!/usr/bin/env python3
"""Benchmark of the PicoSpec verification path on one MI355X.

A step is one full round of the hot path over one batch of synthetic input already resident in HBM:
picospec_compress over all draft rows, picospec_verify over all target rows, picospec_sample_residual
for every sequence.  The default workload is the largest configuration (cfg4: B=256, gamma=16,
V=151,936, fp32, k=4096).  Prints ONE JSON line with the whole-round throughput in verified draft
positions per second, the HBM roofline of the dominant kernel (the compress pass), and the CPU oracle
timed on a bounded sample of the same workload on this machine's host cores.  The timed steps carry one pair
of HIP events each, around the compress call (the kernel the roofline is quoted for); the per-call figures
in `call_ms` come from a few extra steps after the timed region.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth

# HBM traffic of one compress launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), scaled by
# the same counters' reading for a plain copy kernel of known size; see profiles/.  Bytes per launch.
MEASURED_TRAFFIC = {"cfg4": 2.672e9, "cfg5": 1.387e9, "cfg3": 1.364e8}   # profiles/*.md


def algorithmic_bytes(w, N, B):
    """Bytes the method has to move once (the roofline numerator), per call."""
    e = 4 if w.dtype == "f32" else 2
    rec = N * w.k * 8                       # sparse records: int32 id + fp32 prob
    compress = N * w.V * e + rec + N * 12   # rows read once, records + count/mass/lse written once
    verify = (N + B) * w.V * e + rec + (N + B) * 12 + N * 16
    residual = B * (w.V * e + w.k * 8)      # one target row per sequence re-read, one record
    return dict(compress=compress, verify=verify, residual=residual, total=compress + verify + residual)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=30,
                    help="untimed steps first: the first twenty or so rounds after start-up run 5-10 %% slower")
    ap.add_argument("--config", default="cfg4", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--batch", type=int, default=0, help="override the number of sequences (debugging)")
    ap.add_argument("--cpu-seqs", type=int, default=-1, help="sequences in the oracle's timed sample (0 = skip)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (reference for rocprofv3 --pmc byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2603_19133_amd import binding as ps      # raises if the HIP library is not built
    from paper_2603_19133_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs the GPU", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    w = W.WORKLOADS[args.config]
    if args.batch:
        w = w.scaled(B=args.batch)

    t0 = time.time()
    r = W.build_round(w, 0)
    t_gen = time.time() - t0
    B, N = r.B, r.N

    def to_dev(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    draft, tgt = to_dev(r.draft_logits), to_dev(r.tgt_logits)
    seq_off, uni, duni = to_dev(r.seq_off), to_dev(r.uniforms), to_dev(r.draft_uniforms)
    q = ps.alloc_compressed(N, w.k, dev)
    ver = ps.alloc_verified(B, N, dev)
    res = ps.alloc_residual(B, dev)

    # untimed set-up: the drafter's tokens come from the compressed draft distributions
    ps.compress(draft, w.V, w.T, w.k, w.top_p, out=q)
    tok, _ = ps.sample_draft(q, duni)
    torch.cuda.synchronize()

    def step(ev=None, breakdown=False):
        if ev:
            ev[0].record()
        ps.compress(draft, w.V, w.T, w.k, w.top_p, out=q)
        if ev:
            ev[1].record()
        ps.verify(tgt, w.V, w.T, seq_off, N, tok, q, uni, out=ver)
        if breakdown:
            ev[2].record()
        ps.sample_residual(tgt, w.V, w.T, seq_off, N, ver, q, uni, out=res)
        if breakdown:
            ev[3].record()

    if args.copy_probe_mib:
        src = torch.empty(args.copy_probe_mib << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # The timed region: K steps, each with one pair of events around the dominant kernel's call (every event
    # between two kernels costs the round a few microseconds, so the other calls carry none here).
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / args.steps
    compress_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in events]))
    # per-step times from the same events (start of compress to start of the next step's compress)
    step_ms = np.array([events[i][0].elapsed_time(events[i + 1][0]) for i in range(args.steps - 1)]) if args.steps > 1 else np.array([ms_step])

    # After it, outside the timed region: a few more steps with events between all calls, for the per-call figures.
    n_bd = max(1, min(args.steps, 10))
    bd_events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(n_bd)]
    for i in range(n_bd):
        step(bd_events[i], breakdown=True)
    torch.cuda.synchronize()
    call_ms = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(3)] for e in bd_events]).mean(axis=0)

    # The same round through the one-call entry point (three launches at this size: the acceptance test and the
    # residual draw of a sequence share a workgroup), also outside the timed region.
    n_oc = max(1, min(args.steps, 50))
    oc = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ps.round(draft, tgt, w.V, w.T, seq_off, N, tok, w.k, uni, top_p=w.top_p, q=q, ver=ver, res=res)
    oc[0].record()
    for _ in range(n_oc):
        ps.round(draft, tgt, w.V, w.T, seq_off, N, tok, w.k, uni, top_p=w.top_p, q=q, ver=ver, res=res)
    oc[1].record()
    torch.cuda.synchronize()
    one_call_ms = oc[0].elapsed_time(oc[1]) / n_oc

    alg = algorithmic_bytes(w, N, B)
    compress_gbs = alg["compress"] / (compress_ms * 1e-3) / 1e9
    n_acc = ver.n_accept.cpu().numpy()

    out = {
        "metric": "verified draft positions/sec (compress + verify + sample_residual, 1 GPU)",
        "value": N / (ms_step * 1e-3),
        "unit": "positions/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: B={B} gamma={w.gamma_lo}..{w.gamma_hi} V={w.V} {w.dtype} T={w.T} "
                               f"k={w.k} top_p={w.top_p}", "draft_rows": N, "target_rows": N + B,
                   "parallelism": "1 GPU"},
        "round_algorithmic_GBps": alg["total"] / (ms_step * 1e-3) / 1e9,
        "round_frac_of_hbm_peak": alg["total"] / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "step_ms": {"median": float(np.median(step_ms)), "min": float(step_ms.min()), "max": float(step_ms.max())},
        "compress_ms": compress_ms,
        "one_call_ms": one_call_ms,
        "call_ms": {"compress": float(call_ms[0]), "verify": float(call_ms[1]), "sample_residual": float(call_ms[2]),
                    "note": f"{n_bd} extra steps after the timed region, events between all calls"},
        "call_GBps": {"compress": alg["compress"] / (call_ms[0] * 1e-3) / 1e9,
                      "verify": alg["verify"] / (call_ms[1] * 1e-3) / 1e9,
                      "sample_residual": alg["residual"] / (call_ms[2] * 1e-3) / 1e9},
        "mean_accepted": float(n_acc.mean()),
        "input_generation_s": t_gen,
        "roofline": {"kernel": "compress_kernel", "bound": "hbm", "achieved": compress_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": compress_gbs / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC.get(args.config)},
    }

    # the CPU oracle, as it stands, on a bounded sample of the same workload
    n_cpu = args.cpu_seqs if args.cpu_seqs >= 0 else min(B, 256)
    if n_cpu > 0:
        import oracle
        sub = W.build_round(w, 0, seqs=range(n_cpu))
        tok_sub = tok.cpu().numpy()[: sub.N]       # same drafted tokens (prefix of the batch)
        t0 = time.perf_counter()
        oq = oracle.compress(sub.draft_logits, w.V, w.T, w.k, w.top_p)
        ov = oracle.verify(sub.tgt_logits, w.V, w.T, sub.seq_off, tok_sub, oq, sub.uniforms)
        oracle.sample_residual(sub.tgt_logits, w.V, w.T, sub.seq_off, ov.n_accept, ov.tgt_lse, oq, sub.uniforms)
        t_cpu = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": sub.N / t_cpu, "unit": "positions/s", "cores": oracle.threads(),
                               "kind": "oracle",
                               "sample": f"first {n_cpu} sequences of the same round ({sub.N} draft rows, "
                                         f"{sub.N + n_cpu} target rows), {t_cpu:.1f} s"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
