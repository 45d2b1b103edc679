"""Seeded random sweep of picospec_compress against the oracle: vocabulary sizes around the kernel's internal
boundaries (the 8192-element sample, sub-tiles of 4096, the 16-byte vectors), record lengths from 1 to 4096,
both dtypes, temperatures, top-p, rows off the 16-byte boundary, and value patterns that steer the selector
through its passes (plain, heavy-tailed, trending with the id, masked, tie-heavy)."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2603_19133_amd import workloads as W

pytestmark = pytest.mark.gpu

N_CASES = int(os.environ.get("PICOSPEC_SWEEP_CASES", "480"))     # a multiple of 8; raise it for a longer hunt
SEED0 = int(os.environ.get("PICOSPEC_SWEEP_SEED", "0"))          # first seed: move it to hunt on fresh cases


def _case(seed):
    rng = np.random.default_rng(1000 + seed)
    V = int(rng.choice([int(rng.integers(8193, 8300)), int(rng.integers(8300, 12400)), int(rng.integers(12000, 33000)),
                        int(rng.integers(33000, 70000)), 8192 + 4096 * int(rng.integers(1, 6)) + int(rng.integers(-3, 4)),
                        int(rng.integers(2, 8193)), int(rng.integers(100_000, 270_000))]))
    k = int(min(V, 4096, max(1, round(float(np.exp(rng.uniform(0, np.log(4096))))))))
    dtype = str(rng.choice(["f32", "bf16"]))
    T = float(rng.choice([0.3, 0.7, 1.0, 1.0, 1.5, 4.0]))
    top_p = float(rng.choice([0.0, 0.0, 0.5, 0.9, 0.99]))
    shift = int(rng.choice([0, 0, 0, 1, 2, 3, 5]))
    pattern = str(rng.choice(["normal", "zipf", "trend", "head", "masked", "ties", "coarse_values", "few_values", "ramp"]))
    rows = 3
    ld = V + shift
    ids = np.arange(ld, dtype=np.float64)
    z = rng.standard_normal((rows, ld)) * float(rng.choice([0.5, 3.0, 8.0]))
    if pattern == "zipf":
        z = -1.2 * np.log(np.stack([rng.permutation(ld) for _ in range(rows)]) + 1.0) + 0.5 * rng.standard_normal((rows, ld))
    elif pattern == "trend":
        z = z + float(rng.choice([-12.0, -3.0, 3.0, 12.0])) * ids / ld
    elif pattern == "head":
        z = z + np.where(ids < float(rng.choice([300, 4096, 8192, 20000])), float(rng.choice([-8.0, 5.0, 9.0])), 0.0)
    elif pattern == "masked":
        keep = rng.random((rows, ld)) < float(rng.choice([0.5, 0.05, 0.005]))
        keep[:, int(rng.integers(shift, ld))] = True        # a row without any finite logit has no distribution
        z = np.where(keep, z, -np.inf)
    elif pattern == "ties":
        z = np.round(z)
    elif pattern == "coarse_values":
        z = np.round(z * 4) / 4 + 16.0          # few distinct values, all in one binade
    elif pattern == "few_values":               # three to seven distinct values: the k-th largest is shared by very many
        z = np.round(rng.standard_normal((rows, ld)) * float(rng.choice([0.3, 0.5, 0.7, 1.0])))
        if rng.random() < 0.3:
            z = np.where(rng.random((rows, ld)) < 0.02, -np.inf, z)
    elif pattern == "ramp":                     # values that rise or fall along the row in steps, with ties inside a step
        steps = int(rng.choice([3, 17, 200, 5000]))
        z = np.floor(ids * steps / ld)[None, :] * float(rng.choice([-1.0, 1.0])) + np.zeros((rows, 1))
        top_p = 0.0                             # (identical rows: one cumulative sum on the threshold would exclude them all)
    return dict(V=V, k=k, dtype=dtype, T=T, top_p=top_p, shift=shift, pattern=pattern), z.astype(np.float32)


def _pattern_rows(rng, pattern, rows, ld, shift):
    """`rows` rows of one value pattern (the patterns of _case)."""
    ids = np.arange(ld, dtype=np.float64)
    z = rng.standard_normal((rows, ld)) * float(rng.choice([0.5, 3.0, 8.0]))
    if pattern == "zipf":
        z = -1.2 * np.log(np.stack([rng.permutation(ld) for _ in range(rows)]) + 1.0) + 0.5 * rng.standard_normal((rows, ld))
    elif pattern == "trend":
        z = z + float(rng.choice([-12.0, -3.0, 3.0, 12.0])) * ids / ld
    elif pattern == "head":
        z = z + np.where(ids < float(rng.choice([300, 4096, 8192, 20000])), float(rng.choice([-8.0, 5.0, 9.0])), 0.0)
    elif pattern == "masked":
        keep = rng.random((rows, ld)) < float(rng.choice([0.5, 0.05, 0.005]))
        keep[:, int(rng.integers(shift, ld))] = True
        z = np.where(keep, z, -np.inf)
    elif pattern == "ties":
        z = np.round(z)
    elif pattern == "few_values":
        z = np.round(rng.standard_normal((rows, ld)) * float(rng.choice([0.3, 0.5, 0.7, 1.0])))
    elif pattern == "spike":                    # one value far above the rest, where the threshold's sample mostly misses it
        z[np.arange(rows), rng.integers(shift, ld, rows)] = float(rng.choice([90.0, 200.0, 3000.0]))
    return z


N_FULL = int(os.environ.get("PICOSPEC_SWEEP_FULL", "8"))              # calls of more rows than the chip holds at a time


@pytest.mark.parametrize("seed", range(N_FULL))
def test_compress_random_sweep_with_the_chip_full(gpu, seed):
    """Calls of 530-700 rows (more than two workgroups per CU: the kernels that hold the optimistic pass only, with the large
    and with the small candidate buffer, and the launch behind them that takes the rows they give up), the value pattern
    changing every few dozen rows, odd leading dimensions and record lengths across the range."""
    import parity_util as pu
    from paper_2603_19133_amd import binding as ps
    rng = np.random.default_rng(90_000 + SEED0 + seed)
    V = int(rng.choice([int(rng.integers(8300, 12400)), int(rng.integers(12000, 33000)), int(rng.integers(33000, 70000)),
                        int(rng.integers(33000, 70000)), int(rng.integers(100_000, 160_000))]))
    k = int(min(V, 4096, max(1, round(float(np.exp(rng.uniform(np.log(8), np.log(4096))))))))
    dtype = str(rng.choice(["f32", "bf16"]))
    T = float(rng.choice([0.5, 1.0, 1.0, 2.0]))
    shift = int(rng.choice([0, 0, 1, 3]))
    rows, ld = int(rng.integers(530, 700)), V + shift
    parts, left = [], rows
    while left > 0:
        n = min(left, int(rng.integers(20, 80)))
        pattern = str(rng.choice(["normal", "normal", "zipf", "trend", "head", "masked", "ties", "few_values", "spike"]))
        parts.append(_pattern_rows(rng, pattern, n, ld, shift).astype(np.float32))
        left -= n
    z = np.concatenate(parts)
    print("[case] sweep chip full", seed, dict(V=V, k=k, dtype=dtype, T=T, shift=shift, rows=rows), flush=True)
    stored = z if dtype == "f32" else W.to_bf16_bits(z)
    dev = pu.to_device(stored, gpu)
    o = oracle.compress(np.ascontiguousarray(stored[:, shift:]), V, T, k, 0.0)
    g = ps.compress(dev[:, shift:], V, T, k, 0.0)
    torch.cuda.synchronize()
    pu.compare_compress(g, o, 0.0)


@pytest.mark.parametrize("block", range(8))
def test_compress_random_sweep(gpu, block):
    import parity_util as pu
    from paper_2603_19133_amd import binding as ps
    per = N_CASES // 8
    for seed in range(SEED0 + block * per, SEED0 + (block + 1) * per):
        c, z = _case(seed)
        print("[case] sweep", seed, c, flush=True)
        stored = z if c["dtype"] == "f32" else W.to_bf16_bits(z)
        dev = pu.to_device(stored, gpu)
        s = c["shift"]
        o = oracle.compress(np.ascontiguousarray(stored[:, s:]), c["V"], c["T"], c["k"], c["top_p"])
        g = ps.compress(dev[:, s:], c["V"], c["T"], c["k"], c["top_p"])
        torch.cuda.synchronize()
        pu.compare_compress(g, o, c["top_p"])


# ---------------------------------------------------------------- whole rounds

N_ROUNDS = int(os.environ.get("PICOSPEC_SWEEP_ROUNDS", "160"))         # a multiple of 8


def _round_case(seed):
    rng = np.random.default_rng(50_000 + seed)
    big = rng.random() < 0.15                                          # enough rows for picospec_round's three-launch schedule
    B = int(rng.integers(70, 130)) if big else int(rng.integers(1, 13))
    g = rng.integers(0, 7, size=B).astype(np.int32)                    # gamma_b = 0 is legal: only the bonus token
    off = np.zeros(B + 1, np.int32)
    off[1:] = np.cumsum(g)
    N = int(off[-1])
    V = int(rng.choice([int(rng.integers(2, 300)), int(rng.integers(300, 8193)), int(rng.integers(8193, 9000)),
                        int(rng.integers(9000, 36000))]))
    if big:
        V = min(V, int(rng.integers(50, 3000)))
    elif B <= 3 and rng.random() < 0.5:                                # a few sequences over a long vocabulary: many tiles
        V = int(rng.integers(100_000, 300_000))
    k = int(min(V, 1024, max(1, round(float(np.exp(rng.uniform(0, np.log(1024))))))))
    dtype = str(rng.choice(["f32", "bf16"]))
    T = float(rng.choice([0.5, 1.0, 1.0, 2.0]))
    top_p = float(rng.choice([0.0, 0.0, 0.0, 0.9]))
    renorm = int(rng.choice([1, 1, 0]))
    pattern = str(rng.choice(["normal", "zipf", "masked", "peaked"]))
    tgt = rng.standard_normal((N + B, V)) * float(rng.choice([1.0, 3.0]))
    if pattern == "zipf":
        tgt = -1.2 * np.log(np.stack([rng.permutation(V) for _ in range(N + B)]) + 1.0) + 0.5 * tgt
    elif pattern == "peaked":                                          # one token carries almost all of the mass
        tgt[np.arange(N + B), rng.integers(0, V, N + B)] += 14.0
    drows = np.concatenate([np.arange(off[b] + b, off[b] + b + g[b]) for b in range(B)]).astype(np.int64) if N else np.zeros(0, np.int64)
    draft = tgt[drows] * float(rng.choice([1.0, 0.8])) + rng.standard_normal((N, V)) * float(rng.choice([0.0, 0.3, 1.5]))
    if pattern == "masked":                                            # the same mask on both sides, one id always allowed
        keep = rng.random(V) < float(rng.choice([0.5, 0.05]))
        keep[int(rng.integers(0, V))] = True
        tgt = np.where(keep, tgt, -np.inf)
        draft = np.where(keep, draft, -np.inf)
    conv = (lambda a: a.astype(np.float32)) if dtype == "f32" else (lambda a: W.to_bf16_bits(a.astype(np.float32)))
    w = W.Workload(f"sweep{seed}", 99, B, 0, 6, V, dtype, T, k, top_p, 1, "sweep")
    r = W.Round(w, 0, np.arange(B), off, conv(draft).reshape(N, V), conv(tgt), rng.random(N + B, dtype=np.float32),
                rng.random(N, dtype=np.float32))
    return dict(B=B, N=N, V=V, k=k, dtype=dtype, T=T, top_p=top_p, renorm=renorm, pattern=pattern), r, renorm


@pytest.mark.parametrize("block", range(8))
def test_round_random_sweep(gpu, block):
    """Ragged random rounds through the three calls and through picospec_round, against the oracle."""
    import parity_util as pu
    from paper_2603_19133_amd import binding as ps
    per = N_ROUNDS // 8
    for seed in range(SEED0 + block * per, SEED0 + (block + 1) * per):
        c, r, renorm = _round_case(seed)
        print("[case] round sweep", seed, c, flush=True)
        o = pu.oracle_round(r, renorm=renorm)
        pu.compare_round(pu.gpu_round(r, o.tok, gpu, renorm=renorm), o, r, max_excluded_frac=0.34, strict=False)
        pu.compare_round(pu.gpu_round(r, o.tok, gpu, renorm=renorm, seg=True), o, r, max_excluded_frac=0.34, strict=False)
        d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(gpu)
        w = r.workload
        q, ver, res = ps.round(pu.to_device(r.draft_logits, gpu), pu.to_device(r.tgt_logits, gpu), w.V, w.T, d(r.seq_off),
                               r.N, d(o.tok), w.k, d(r.uniforms), top_p=w.top_p, renorm=renorm)
        torch.cuda.synchronize()
        pu.compare_round(pu.GpuRound(q, ver, res), o, r, max_excluded_frac=0.34, strict=False)


@pytest.mark.parametrize("block", range(4))
def test_downlink_and_ranges_random_sweep(gpu, block):
    """The same random rounds through the paper's own downlink (record of the rejected target row, local
    resampling at the edge) and through the verification of three consecutive ranges of positions."""
    import parity_util as pu
    import test_gpu_downlink as D
    import test_gpu_verify_range as VR
    from paper_2603_19133_amd import binding as ps
    per = N_ROUNDS // 8
    for seed in range(SEED0 + block * per, SEED0 + (block + 1) * per):
        c, r, renorm = _round_case(7000 + seed)
        print("[case] downlink/ranges sweep", seed, c, flush=True)
        w = r.workload
        D._downlink(pu, ps, gpu, r, min(w.k, w.V), renorm, strict=False)
        VR._ranges_case(pu, ps, gpu, r, w.k, seed)


@pytest.mark.parametrize("block", range(2))
def test_wire_random_sweep(gpu, block):
    """Random batches of records through the downlink message (bytes against the oracle's, every format, receivers
    with as many or fewer slots) and random drafts through the uplink message."""
    import parity_util as pu
    import test_gpu_wire as Wt
    from paper_2603_19133_amd import binding as ps
    per = N_ROUNDS // 4
    for seed in range(SEED0 + block * per, SEED0 + (block + 1) * per):
        rng = np.random.default_rng(90_000 + seed)
        B, k, gmax = int(rng.integers(0, 70)), int(rng.integers(1, 300)), int(rng.integers(0, 17))
        fmt = int(rng.integers(0, 3))
        print("[case] wire sweep", seed, dict(B=B, k=k, gmax=gmax, fmt=fmt), flush=True)
        seq_off, n_accept, token, idx, prob, count = Wt._batch(seed, B, k, gmax=gmax, tiny=bool(seed % 3 == 0))
        want, n = oracle.pack_downlink(seq_off, n_accept, token, idx, prob, count, fmt)
        d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(gpu)
        cap = ps.downlink_bytes_max(B, k, fmt)
        wire = torch.full((cap + 8,), 0xEE, dtype=torch.uint8, device=gpu)
        _, nbytes, status = ps.pack_downlink(d(seq_off), d(n_accept), d(token), Wt._rec(ps, gpu, idx, prob, count), fmt, wire=wire)
        torch.cuda.synchronize()
        got = wire.cpu().numpy()
        assert int(nbytes.item()) == n and int(status.item()) == 0
        assert np.array_equal(got[:n], want) and np.all(got[n:] == 0xEE)
        for k2 in sorted({k, max(1, k // 3)}):
            Wt._compare_unpacked(pu, ps.unpack_downlink(d(want), n, B, k2), oracle.unpack_downlink(want, B, k2), k2)
        # uplink of the same ragged shape
        N = int(seq_off[-1])
        tok = rng.integers(0, 152064, N).astype(np.int32)
        q = np.exp2(rng.uniform(-28, 0, N)).astype(np.float32)
        wantu, nu = oracle.pack_uplink(seq_off, tok, q, fmt)
        wu = torch.full((nu + 8,), 0xEE, dtype=torch.uint8, device=gpu)
        _, nb = ps.pack_uplink(d(seq_off), N, d(tok), d(q), fmt, wire=wu)
        torch.cuda.synchronize()
        gotu = wu.cpu().numpy()
        assert int(nb.item()) == nu and np.array_equal(gotu[:nu], wantu) and np.all(gotu[nu:] == 0xEE)
        n_max = int(rng.integers(0, N + 3))
        o = oracle.unpack_uplink(wantu, B, n_max)
        so, t, qq, st = ps.unpack_uplink(d(wantu), nu, B, n_max)
        torch.cuda.synchronize()
        kept = int(o.seq_off[-1])
        assert int(st.item()) == o.status and np.array_equal(pu.n(so), o.seq_off)
        assert np.array_equal(pu.n(t)[:kept], o.draft_tok[:kept]) and np.array_equal(pu.n(qq)[:kept].astype(np.float64), o.q_scalar[:kept])


def test_sample_draft_random_sweep(gpu):
    """The drafter's draw over records of random lengths (1 to 5000 slots, rows on and off 16-byte boundaries)."""
    import parity_util as pu
    import test_gpu_parity as P
    from paper_2603_19133_amd import binding as ps
    for seed in range(SEED0, SEED0 + N_ROUNDS // 2):
        rng = np.random.default_rng(120_000 + seed)
        k = int(min(5000, max(1, round(float(np.exp(rng.uniform(0, np.log(5000))))))))
        print("[case] sample_draft sweep", seed, k, flush=True)
        P._sample_draft_case(gpu, pu, ps, k, 120_000 + seed)
