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

The timed rounds are consecutive and every one has uniforms of its own, prepared on the device beforehand.  The
smaller configurations cycle through several resident input sets so that no round finds its logits in the caches;
cfg5 (ragged asynchronous rounds) runs its 100 consecutive rounds over eight resident rounds of the workload (rounds
0..7, each with its own draft lengths and row packing: all 100 would need 280 GB of logits).
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

# HBM traffic of one compress launch (bytes), a constant taken from the rocprofv3 --pmc runs summarised under
# profiles/ (FETCH_SIZE and WRITE_SIZE, scaled by the same counters' reading for a plain copy of known size): it is
# NOT measured in this run, and the JSON line says so next to it.
PROFILED_TRAFFIC = {"cfg4": (2.672e9, "profiles/cfg4_round_kernels.md"), "cfg5": (1.401e9, "profiles/cfg5_cfg3_round_kernels.md"),
                    "cfg3": (1.364e8, "profiles/cfg5_cfg3_round_kernels.md")}
# distinct resident input sets a run cycles through, so that no step finds its logits in the caches (cfg4's single set
# is 22 times the 256 MB Infinity Cache); cfg5's sets are rounds 0..7 of the workload, each with its own draft lengths
DEFAULT_SETS = {"cfg1": 8, "cfg2": 8, "cfg3": 4, "cfg4": 1, "cfg5": 8}
DEFAULT_STEPS = {"cfg5": 100}            # the workload's 100 consecutive rounds


def algorithmic_bytes(w, N, B, seg_table_bytes=0):
    """Bytes the method has to move once (the roofline numerator), per call.  With the segment table the draw does not
    read its target row again: it reads the record, one gathered logit per record entry, its row of the table and one
    segment of at most 4 KB; the table itself is written once by verify."""
    e = 4 if w.dtype == "f32" else 2
    rec = N * w.k * 8                       # sparse records: int32 id + fp32 prob
    compress = N * w.V * e + rec + N * 12   # rows read once, records + count/mass/lse written once
    verify = (N + B) * w.V * e + rec + (N + B) * 12 + N * 16 + seg_table_bytes
    if seg_table_bytes:
        residual = B * (w.k * 8 + w.k * e + 4096 + seg_table_bytes // max(1, N + B))
    else:
        residual = B * (w.V * e + w.k * 8)  # one target row per sequence re-read, one record
    return dict(compress=compress, verify=verify, residual=residual, total=compress + verify + residual)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed rounds (default 200; cfg5: its 100 consecutive rounds)")
    ap.add_argument("--warmup", type=int, default=30,
                    help="untimed steps first: the first twenty or so rounds after start-up run 5-10 %% slower")
    ap.add_argument("--settle-ms", type=float, default=60.0,
                    help="before the warm-up steps: untimed rounds for this many milliseconds, so that the device has left the dip "
                         "of its effective shader clock that follows every pause (3-40 ms after work resumes; --burst shows it) "
                         "whatever --warmup is; 0 switches it off")
    ap.add_argument("--config", default="cfg4", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--batch", type=int, default=0, help="override the number of sequences (debugging)")
    ap.add_argument("--sets", type=int, default=0, help="distinct resident input sets to cycle through (default per config)")
    ap.add_argument("--cpu-seqs", type=int, default=-1, help="sequences in the oracle's timed sample (0 = skip)")
    ap.add_argument("--burst", type=int, default=0,
                    help="instead of the benchmark: after --burst-idle seconds of pause, this many compress calls back to back, "
                         "each followed by a clock probe; prints the per-call duration and the shader clock behind it")
    ap.add_argument("--burst-idle", type=float, default=2.0)
    ap.add_argument("--no-workspace", action="store_true",
                    help="run verify / sample_residual without the optional workspace (the draw then streams its target row again)")
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

    steps = args.steps or DEFAULT_STEPS.get(args.config, 200)
    n_sets = max(1, args.sets or DEFAULT_SETS[args.config])
    n_sets = min(n_sets, steps)

    def to_dev(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    # Input sets, all resident in HBM before anything is timed.  Set i is round i of the workload (cfg5: its own draft
    # lengths, hence its own packing of the rows; the fixed-length workloads: the same logits in buffers of their own).
    class InputSet:
        pass

    t0 = time.time()
    sets = []
    for i in range(n_sets):
        r = W.build_round(w, i)
        x = InputSet()
        x.round, x.B, x.N = r, r.B, r.N
        x.draft, x.tgt = to_dev(r.draft_logits), to_dev(r.tgt_logits)
        x.seq_off, x.duni = to_dev(r.seq_off), to_dev(r.draft_uniforms)
        x.q = ps.alloc_compressed(r.N, w.k, dev)
        x.ver = ps.alloc_verified(r.B, r.N, dev)
        x.res = ps.alloc_residual(r.B, dev)
        x.ws = None if args.no_workspace else ps.alloc_workspace(x.tgt.dtype, r.N + r.B, w.V, dev, ps.CALL_ROUND)
        x.ws_bytes = 0 if x.ws is None else x.ws.numel()
        # untimed set-up: the drafter's tokens come from the compressed draft distributions
        ps.compress(x.draft, w.V, w.T, w.k, w.top_p, out=x.q)
        x.tok, _ = ps.sample_draft(x.q, x.duni)
        if i:
            x.round = None                   # (the host copy of set 0 alone is needed again, for round 0's uniforms)
        sets.append(x)
    torch.cuda.synchronize()
    t_gen = time.time() - t0
    B, N = sets[0].B, sets[0].N
    # every timed round has uniforms of its own (round i of the workload's stream, cut to the set's row count)
    gen = torch.Generator(device=dev)
    gen.manual_seed(W.BASE_SEED + 7)
    uniforms = [torch.rand(sets[i % n_sets].N + sets[i % n_sets].B, device=dev, generator=gen) for i in range(steps)]
    uniforms[0] = to_dev(sets[0].round.uniforms)          # (round 0 exactly as the parity tests see it)
    torch.cuda.synchronize()

    def step(i, ev=None, breakdown=False):
        x, uni = sets[i % n_sets], uniforms[i % steps]
        if ev:
            ev[0].record()
        ps.compress(x.draft, w.V, w.T, w.k, w.top_p, out=x.q)
        if ev:
            ev[1].record()
        ps.verify(x.tgt, w.V, w.T, x.seq_off, x.N, x.tok, x.q, uni, out=x.ver, workspace=x.ws)
        if breakdown:
            ev[2].record()
        ps.sample_residual(x.tgt, w.V, w.T, x.seq_off, x.N, x.ver, x.q, uni, out=x.res, workspace=x.ws)
        if breakdown:
            ev[3].record()

    if args.burst:
        # Where the slow first rounds come from: after a pause the device's effective shader clock dips for some tens
        # of milliseconds (the compress kernel is bound by the vector ALU and follows it).
        x = sets[0]
        n = args.burst
        ticks = torch.zeros((n, 2), dtype=torch.int64, device=dev)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n)]
        torch.cuda.synchronize()
        time.sleep(args.burst_idle)
        for i in range(n):
            ev[i][0].record()
            ps.compress(x.draft, w.V, w.T, w.k, w.top_p, out=x.q)
            ev[i][1].record()
            ps.probe_clock(ticks[i])
        torch.cuda.synchronize()
        tk = ticks.cpu().numpy().astype(np.float64)
        print(f"# {w.name}: {n} compress calls back to back after {args.burst_idle} s of pause")
        print("# call  start_ms  compress_us  shader_clock_MHz")
        for i in range(n):
            print(f"{i:5d}  {ev[0][0].elapsed_time(ev[i][0]):8.2f}  {ev[i][0].elapsed_time(ev[i][1]) * 1e3:11.1f}  {100.0 * tk[i, 0] / tk[i, 1]:8.0f}")
        return 0

    if args.copy_probe_mib:
        src = torch.empty(args.copy_probe_mib << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    clock_ticks = torch.zeros((2, 2), dtype=torch.int64, device=dev)
    # Settling (untimed, reported in the JSON line): the device was idle while the inputs were made, and for some tens of
    # milliseconds after work resumes its effective shader clock dips, which the compress kernel follows.  The rounds
    # here keep it busy through that; the warm-up steps follow without a pause.
    settled_rounds = 0
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for _ in range(4):
            step(settled_rounds)
            settled_rounds += 1
        torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i)
    ps.probe_clock(clock_ticks[0])           # the shader clock at the start of the timed region ...
    torch.cuda.synchronize()
    # The timed region: K consecutive rounds, each with one pair of events around the dominant kernel's call (every
    # event between two kernels costs the round a few microseconds, so the other calls carry none here).
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        step(i, events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ps.probe_clock(clock_ticks[1])           # ... and at its end
    torch.cuda.synchronize()
    ck = clock_ticks.cpu().numpy().astype(np.float64)
    clock_mhz = [float(100.0 * ck[j, 0] / ck[j, 1]) for j in range(2)]
    ms_step = wall * 1e3 / steps
    n_timed = sum(sets[i % n_sets].N for i in range(steps))               # draft positions verified in the timed region
    compress_each = np.array([e[0].elapsed_time(e[1]) for e in events])
    compress_ms = float(compress_each.mean())
    # per-step times from the same events (start of compress to start of the next step's compress)
    step_ms = np.array([events[i][0].elapsed_time(events[i + 1][0]) for i in range(steps - 1)]) if steps > 1 else np.array([ms_step])

    # After it, outside the timed region: a few more steps with events between all calls, for the per-call figures.
    n_bd = max(1, min(steps, 10))
    bd_events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(n_bd)]
    for i in range(n_bd):
        step(i, bd_events[i], breakdown=True)
    torch.cuda.synchronize()
    call_ms = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(3)] for e in bd_events]).mean(axis=0)

    # The same rounds through the one-call entry point (three launches at the large sizes: the acceptance test and the
    # residual draw of a sequence share a workgroup), also outside the timed region.
    n_oc = max(1, min(steps, 50))
    oc = [torch.cuda.Event(enable_timing=True) for _ in range(2)]

    def one_call(i):
        x = sets[i % n_sets]
        ps.round(x.draft, x.tgt, w.V, w.T, x.seq_off, x.N, x.tok, w.k, uniforms[i % steps], top_p=w.top_p, q=x.q, ver=x.ver, res=x.res,
                 workspace=x.ws)

    one_call(0)
    oc[0].record()
    for i in range(n_oc):
        one_call(i)
    oc[1].record()
    torch.cuda.synchronize()
    one_call_ms = oc[0].elapsed_time(oc[1]) / n_oc

    # algorithmic bytes: of the timed region (the sets differ in their row counts) and of the breakdown steps
    alg_steps = [algorithmic_bytes(w, sets[i % n_sets].N, sets[i % n_sets].B, sets[i % n_sets].ws_bytes) for i in range(steps)]
    alg_total = sum(a["total"] for a in alg_steps)
    alg_compress = sum(a["compress"] for a in alg_steps)
    alg_bd = {k: float(np.mean([algorithmic_bytes(w, sets[i % n_sets].N, sets[i % n_sets].B, sets[i % n_sets].ws_bytes)[k] for i in range(n_bd)]))
              for k in ("compress", "verify", "residual")}
    compress_gbs = alg_compress / (compress_each.sum() * 1e-3) / 1e9
    n_acc = sets[0].ver.n_accept.cpu().numpy()
    set_bytes = (sets[0].draft.numel() + sets[0].tgt.numel()) * sets[0].draft.element_size()
    cache_resident = n_sets * set_bytes < 2 * 256e6          # (all sets together within reach of the 256 MB Infinity Cache)
    traffic = PROFILED_TRAFFIC.get(args.config)
    head = max(1, min(5, steps // 4))

    out = {
        "metric": "verified draft positions/sec (compress + verify + sample_residual, 1 GPU)",
        "value": n_timed / (wall),
        "unit": "positions/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: B={B} gamma={w.gamma_lo}..{w.gamma_hi} V={w.V} {w.dtype} T={w.T} "
                               f"k={w.k} top_p={w.top_p}", "draft_rows": N if n_sets == 1 else [x.N for x in sets],
                   "target_rows": N + B if n_sets == 1 else [x.N + x.B for x in sets],
                   "input_sets": n_sets, "segment_table": not args.no_workspace, "protocol": f"{steps} consecutive rounds over {n_sets} resident input set(s), "
                   "uniforms of its own for every round" + (f"; {settled_rounds} untimed rounds ({args.settle_ms:g} ms) in front of the "
                   "warm-up steps carry the device through the clock dip that follows a pause" if settled_rounds else ""),
                   "settle_ms": args.settle_ms, "settle_rounds": settled_rounds, "parallelism": "1 GPU"},
        "round_algorithmic_GBps": alg_total / wall / 1e9,
        "round_frac_of_hbm_peak": None if cache_resident else alg_total / wall / 1e9 / HBM_PEAK_GBS,
        "cache_resident": bool(cache_resident),
        "step_ms": {"median": float(np.median(step_ms)), "min": float(step_ms.min()), "max": float(step_ms.max())},
        "compress_ms": compress_ms,
        "compress_ms_first_last": {"first": float(compress_each[:head].mean()), "last": float(compress_each[-head:].mean()),
                                   "note": f"mean of the first and of the last {head} timed rounds: for some tens of milliseconds after a "
                                           "pause the device's effective shader clock dips (bench.py --burst shows it)"},
        "shader_clock_mhz": {"before_timed": clock_mhz[0], "after_timed": clock_mhz[1],
                             "note": "s_memtime / s_memrealtime over a fixed loop (picospec_probe_clock)"},
        "one_call_ms": one_call_ms,
        "call_ms": {"compress": float(call_ms[0]), "verify": float(call_ms[1]), "sample_residual": float(call_ms[2]),
                    "note": f"{n_bd} extra steps after the timed region, events between all calls"},
        "call_GBps": {"compress": alg_bd["compress"] / (call_ms[0] * 1e-3) / 1e9,
                      "verify": alg_bd["verify"] / (call_ms[1] * 1e-3) / 1e9,
                      "sample_residual": alg_bd["residual"] / (call_ms[2] * 1e-3) / 1e9},
        "mean_accepted": float(n_acc.mean()),
        "input_generation_s": t_gen,
        "roofline": {"kernel": "compress_kernel", "bound": "hbm", "achieved": compress_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": compress_gbs / HBM_PEAK_GBS,
                     "traffic": traffic[0] if traffic else None,
                     "traffic_source": (traffic[1] + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this "
                                        "command; a constant here, not measured in this run)") if traffic else None},
    }

    # the CPU oracle, as it stands, on a bounded sample of the same workload
    n_cpu = args.cpu_seqs if args.cpu_seqs >= 0 else min(B, 256)
    if n_cpu > 0:
        import oracle
        sub = W.build_round(w, 0, seqs=range(n_cpu))
        tok_sub = sets[0].tok.cpu().numpy()[: sub.N]       # same drafted tokens (prefix of the batch)
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
