"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element, on the
same seeded inputs (criteria in parity_util)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_19133_amd import workloads as W

pytestmark = pytest.mark.gpu


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


# ---------------------------------------------------------------- the five workloads (full or scaled to oracle speed)

WORKLOAD_CASES = [
    ("cfg1", {}, 0),
    ("cfg2", {}, 0),
    ("cfg3", {"B": 6}, 0),
    ("cfg4", {"B": 3}, 0),
    ("cfg5", {"B": 10}, 0),
    ("cfg5", {"B": 10}, 1),
]


@pytest.mark.parametrize("seg", [False, True])       # without / with the segment table of the target rows
@pytest.mark.parametrize("name,scale,rnd", WORKLOAD_CASES)
def test_round_matches_oracle(gpu, pu, name, scale, rnd, seg):
    w = W.WORKLOADS[name]
    if scale:
        w = w.scaled(**scale)
    _announce("round", name, scale, "round", rnd, "V", w.V, "k", w.k, w.dtype)
    r = W.build_round(w, rnd)
    o = pu.oracle_round(r)
    g = pu.gpu_round(r, o.tok, gpu, seg=seg)
    st = pu.compare_round(g, o, r)
    print("[stats]", name, "seg" if seg else "", {k: v for k, v in st.items() if k != "topp_excluded"}, flush=True)
    if name in ("cfg1", "cfg2", "cfg3"):
        assert st["mismatch_accept"] == 0 and st["mismatch_draw"] == 0


# ---------------------------------------------------------------- compress edge cases

def _compress_case(pu, ps, gpu, z, V, T, k, top_p=0.0, dtype="f32"):
    stored = z if dtype == "f32" else W.to_bf16_bits(z)
    o = oracle.compress(stored, V, T, k, top_p)
    g = ps.compress(pu.to_device(stored, gpu), V, T, k, top_p)
    torch.cuda.synchronize()
    return pu.compare_compress(g, o, top_p)


@pytest.mark.parametrize("V,k", [(1, 1), (8, 8), (8, 3), (63, 1), (1000, 1000), (4096, 4096), (5000, 4096),
                                 (16384, 64), (16385, 64), (32769, 500), (70001, 4096),
                                 (151936, 10), (128256, 1), (40000, 3), (9000, 10), (8193, 30)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_compress_sizes_and_tails(gpu, pu, ps, V, k, dtype):
    _announce("compress sizes", V, k, dtype)
    rng = np.random.default_rng(V * 31 + k)
    z = (rng.standard_normal((5, V)) * 3).astype(np.float32)
    _compress_case(pu, ps, gpu, z, V, 0.9, k, dtype=dtype)


@pytest.mark.parametrize("pattern", ["ties", "all_equal", "ascending", "descending", "neg_inf", "signed_zero",
                                     "two_values", "sawtooth", "trend_down", "trend_up", "head_hot", "head_cold",
                                     "hot_cluster", "period_of_the_sample", "masked_3pct", "masked_block", "masked_few",
                                     "masked_half", "spike"])
# (three rows: the general kernel at two record lengths; 600 rows of a short record on long rows: the variant with three
#  workgroups per CU, which leaves the rows its optimistic pass cannot take to a second launch of the general kernel)
@pytest.mark.parametrize("R,k", [(3, 777), (3, 2500), (600, 777)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_compress_adversarial_rows(gpu, pu, ps, pattern, dtype, R, k):
    _announce("compress adversarial", pattern, dtype, R, k)
    V = 40000
    rng = np.random.default_rng(5)
    if pattern == "ties":
        z = rng.integers(-6, 7, (R, V)).astype(np.float32)
    elif pattern == "all_equal":
        z = np.full((R, V), 1.5, np.float32)
    elif pattern == "ascending":        # defeats the running threshold: every element is admitted
        z = np.tile(np.linspace(-8, 8, V, dtype=np.float32), (R, 1))
    elif pattern == "descending":
        z = np.tile(np.linspace(8, -8, V, dtype=np.float32), (R, 1))
    elif pattern == "neg_inf":
        z = np.where(rng.random((R, V)) < 0.99, -np.inf, rng.standard_normal((R, V))).astype(np.float32)
    elif pattern == "signed_zero":
        z = np.where(rng.random((R, V)) < 0.5, -0.0, 0.0).astype(np.float32)
        z[:, ::97] = -1.0
    elif pattern == "two_values":
        z = np.where(rng.random((R, V)) < 0.01, 2.0, -2.0).astype(np.float32)
    elif pattern == "sawtooth":
        z = np.tile((np.arange(V) % 1000).astype(np.float32) * 0.01, (R, 1))
    elif pattern == "spike":
        # one value per row far above all others, at an id that the threshold's sample sees in some rows and misses in
        # most: the optimistic pass sums exponentials against the sample's largest value and must give such a row up
        z = (rng.standard_normal((R, V)) * 3).astype(np.float32)
        z[np.arange(R), (np.arange(R) * 6151 + 1234) % V] = 160.0
    elif pattern.startswith("masked"):
        # vocabulary masks (-inf everywhere but on the allowed ids): more allowed ids than k, fewer than k (the record
        # is then filled up with masked ids in ascending order), a block of ids, half of the vocabulary
        z = (rng.standard_normal((R, V)) * 3).astype(np.float32)
        ids = np.arange(V)
        allowed = {"masked_3pct": rng.random((R, V)) < 0.03, "masked_few": rng.random((R, V)) < 0.002,
                   "masked_block": np.tile((ids >= 20000) & (ids < 21500), (R, 1)),
                   "masked_half": rng.random((R, V)) < 0.5}[pattern]
        z = np.where(allowed, z, -np.inf).astype(np.float32)
    else:
        # values that depend on the vocabulary id, as logits do (frequent tokens sit at low ids): the threshold
        # comes from a sample spread over the row, and whatever the sample misses the count at the row's end catches
        ids = np.arange(V, dtype=np.float64)
        bias = {"trend_down": -9.0 * ids / V, "trend_up": 9.0 * ids / V,
                "head_hot": np.where(ids < 8192, 6.0, 0.0), "head_cold": np.where(ids < 8192, -6.0, 0.0),
                "hot_cluster": np.where((ids > 20000) & (ids < 20600), 9.0, 0.0),       # between the sample's runs or on them
                "period_of_the_sample": 4.0 * np.cos(2 * np.pi * ids * 256 / V)}[pattern]
        z = (rng.standard_normal((R, V)) * 3 + bias).astype(np.float32)
    _compress_case(pu, ps, gpu, z, V, 1.3, k, dtype=dtype)


@pytest.mark.parametrize("V,k,scale", [(10108, 1400, 0.5), (10108, 1700, 0.5), (12300, 2000, 0.5), (16500, 3000, 0.5),
                                       (36000, 1400, 0.5), (40108, 2000, 0.5), (33000, 700, 0.5)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_compress_ties_at_the_cut_when_the_buffer_fills_in_mid_sub_tile(gpu, pu, ps, V, k, scale, dtype):
    """Rows of a few distinct values whose k-th largest is shared by hundreds of entries, of a length at which
    the candidate buffer fills while the last sub-tiles are appended: the waves of a sub-tile append in any order,
    so the ties that wait through a prune must still be able to displace kept ones with higher ids."""
    _announce("compress ties at the cut", V, k, scale, dtype)
    rng = np.random.default_rng(V + k)
    z = np.round(rng.standard_normal((16, V)) * scale).astype(np.float32)
    _compress_case(pu, ps, gpu, z, V, 1.5, k, dtype=dtype)


@pytest.mark.parametrize("shift", [1, 2, 3, 5])
@pytest.mark.parametrize("V", [20001, 50001])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_compress_unaligned_rows(gpu, pu, ps, shift, dtype, V):
    """Row starts that are not 16-byte aligned (odd leading dimension, offset base pointer)."""
    _announce("compress unaligned", shift, dtype, V)
    ld, k = V + shift, 300
    rng = np.random.default_rng(shift)
    full = (rng.standard_normal((4, ld)) * 2).astype(np.float32)
    stored = full if dtype == "f32" else W.to_bf16_bits(full)
    o = oracle.compress(stored, V, 1.0, k)
    dev = pu.to_device(stored, gpu)
    assert dev.stride(0) == ld
    g = ps.compress(dev, V, 1.0, k)
    pu.compare_compress(g, o)
    # the same rows seen through a base pointer moved by `shift` elements
    o2 = oracle.compress(np.ascontiguousarray(stored[:, shift:]), V - shift, 1.0, k)
    g2 = ps.compress(dev[:, shift:], V - shift, 1.0, k)
    torch.cuda.synchronize()
    pu.compare_compress(g2, o2)


@pytest.mark.parametrize("pattern", ["trend", "masked_above_k", "masked_below_k", "few_values", "mixed"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_compress_every_pass_with_the_chip_full(gpu, pu, ps, pattern, dtype):
    """1100 rows (two generations of workgroups, look-ahead loads live) of the kinds that steer the selector through
    its other passes: values that trend with the id, masks that leave more or fewer ids than k, rows of a few
    distinct values whose buffer fills, and all of them mixed row by row."""
    _chip_full_case(gpu, pu, ps, pattern, dtype, 1100, 12300, 600)


@pytest.mark.parametrize("pattern", ["trend", "masked_above_k", "masked_below_k", "few_values", "mixed"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_compress_every_pass_with_the_chip_full_short_records(gpu, pu, ps, pattern, dtype):
    """The same through the kernel's variant for short records on long rows (three workgroups per CU)."""
    _chip_full_case(gpu, pu, ps, pattern, dtype, 1100, 40000, 600)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_compress_every_pass_at_full_size(gpu, pu, ps, dtype):
    """The same mixture at the largest configuration's row length and record length (600 rows)."""
    _chip_full_case(gpu, pu, ps, "mixed", dtype, 600, 151936, 4096)


def _chip_full_case(gpu, pu, ps, pattern, dtype, rows, V, k):
    _announce("compress chip full", pattern, dtype, rows, V, k)
    rng = np.random.default_rng(len(pattern))
    ids = np.arange(V, dtype=np.float64)
    base = rng.standard_normal((rows, V)) * 3

    def make(p, z):
        if p == "trend":
            return z + 9.0 * ids / V * rng.choice([-1.0, 1.0], (z.shape[0], 1))
        if p == "masked_above_k":
            return np.where(rng.random(z.shape) < 0.15, z, -np.inf)
        if p == "masked_below_k":
            return np.where(rng.random(z.shape) < 0.01, z, -np.inf)
        return np.round(z / 6.0)                                   # few_values: five to seven levels

    if pattern == "mixed":
        kinds = ["trend", "masked_above_k", "masked_below_k", "few_values"]
        z = np.concatenate([make(kinds[i % 4], base[i:i + 1]) for i in range(rows)])
    else:
        z = make(pattern, base)
    z[:, 0] = np.where(np.isfinite(z[:, 0]), z[:, 0], 0.0)          # (no row without a finite entry)
    _compress_case(pu, ps, gpu, z.astype(np.float32), V, 1.0, k, dtype=dtype)


@pytest.mark.parametrize("shape", [(1237, 9001, 9003, 70), (1741, 33001, 33003, 70)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_compress_more_rows_than_resident_workgroups(gpu, pu, ps, dtype, shape):
    """More rows than the chip holds at a time (the look-ahead loads of the next generation of rows are
    live), odd leading dimension so that most rows start off a 16-byte boundary, and a row count that is
    not a multiple of anything; also the same through the row statistics."""
    _announce("compress many rows", dtype, shape)
    rows, V, ld, k = shape
    rng = np.random.default_rng(12)
    full = (rng.standard_normal((rows, ld)) * 3).astype(np.float32)
    stored = full if dtype == "f32" else W.to_bf16_bits(full)
    o = oracle.compress(stored, V, 0.8, k)
    dev = pu.to_device(stored, gpu)
    g = ps.compress(dev, V, 0.8, k)
    mx, sm, ls = ps.row_stats(dev, V, 0.8)
    torch.cuda.synchronize()
    pu.compare_compress(g, o)
    pu.assert_close(pu.n(ls), o.lse, pu.RTOL_LSE, "row_stats lse", atol=2e-6)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows", [700, 1237, 2300])
def test_row_stats_launch_shapes(gpu, pu, ps, dtype, rows):
    """The row statistics pick their workgroup size from the row count and the dtype: every shape gives
    the oracle's max, sum and lse (rows off the 16-byte boundary, ragged tails, a few -inf entries)."""
    _announce("row_stats shapes", dtype, rows)
    V, ld, T = 5003, 5005, 0.9
    rng = np.random.default_rng(rows)
    full = (rng.standard_normal((rows, ld)) * 4).astype(np.float32)
    full[::7, 11] = -np.inf
    stored = full if dtype == "f32" else W.to_bf16_bits(full)
    o = oracle.compress(stored, V, T, 1)
    mx, sm, ls = ps.row_stats(pu.to_device(stored, gpu), V, T)
    torch.cuda.synchronize()
    z = (stored if dtype == "f32" else W.bf16_bits_to_f32(stored)).astype(np.float64)[:, :V]
    assert np.array_equal(pu.n(mx).astype(np.float64), z.max(axis=1))
    pu.assert_close(pu.n(ls), o.lse, pu.RTOL_LSE, "row_stats lse", atol=2e-6)
    pu.assert_close(pu.n(sm), np.exp(o.lse - z.max(axis=1) / T), 1e-5, "row_stats sum")


@pytest.mark.parametrize("tau,k", [(0.5, 512), (0.9, 2048), (0.95, 64), (0.999, 4096)])
def test_compress_top_p(gpu, pu, ps, tau, k):
    _announce("compress top-p", tau, k)
    w = W.WORKLOADS["cfg5"]
    z = np.stack([W.target_row(w, b, 0) for b in range(6)])
    st = _compress_case(pu, ps, gpu, z, w.V, 1.0, k, top_p=tau, dtype="bf16")
    assert not st["topp_excluded"]


def test_compress_zero_rows_and_determinism(gpu, pu, ps):
    _announce("compress zero rows / determinism")
    empty = torch.empty((0, 100), dtype=torch.float32, device=gpu)
    out = ps.compress(empty, 100, 1.0, 10)
    assert out.idx.shape == (0, 10)
    w = W.WORKLOADS["cfg3"]
    z = pu.to_device(W.to_bf16_bits(np.stack([W.target_row(w, 0, t) for t in range(4)])), gpu)
    a = ps.compress(z, w.V, w.T, w.k)
    b = ps.compress(z, w.V, w.T, w.k)
    torch.cuda.synchronize()
    for x, y in ((a.idx, b.idx), (a.prob, b.prob), (a.mass, b.mass), (a.lse, b.lse), (a.count, b.count)):
        assert torch.equal(x, y)


# ---------------------------------------------------------------- verification / residual special cases

def _custom_round(w, draft, tgt, off, uni, duni):
    return W.Round(w, 0, np.arange(len(off) - 1), off, draft, tgt, uni, duni)


def test_identical_distributions_accept_everything(gpu, pu):
    _announce("identical distributions")
    w = W.Workload("ident", 90, 5, 3, 3, 5000, "f32", 1.0, 4096, 0.0, 1, "normal3")
    rng = np.random.default_rng(21)
    g = np.array([3, 1, 0, 4, 2], np.int32)
    off = W.seq_offsets(g)
    N, B = int(off[-1]), 5
    tgt = (rng.standard_normal((N + B, w.V)) * 3).astype(np.float32)
    draft = np.concatenate([tgt[off[b] + b: off[b] + b + g[b]] for b in range(B)])
    # uncompressed limit (k = V): qhat is the full draft distribution, equal to the target's
    w2 = W.Workload("ident", 90, 5, 3, 3, 3000, "f32", 1.0, 3000, 0.0, 1, "normal3")
    r2 = _custom_round(w2, np.ascontiguousarray(draft[:, :3000]), np.ascontiguousarray(tgt[:, :3000]), off,
                       rng.random(N + B, dtype=np.float32), rng.random(N, dtype=np.float32))
    o = pu.oracle_round(r2)
    gq = pu.gpu_round(r2, o.tok, gpu)
    na = pu.n(gq.ver.n_accept)
    # p and qhat are equal up to rounding, so p/qhat straddles 1; only uniforms within rounding of 1 could reject
    assert (na == g).all() and (o.ver.n_accept == g).all()
    assert np.allclose(pu.n(gq.res.resid_mass), 1.0, rtol=1e-5)
    keep = o.res.cdf_margin >= pu.CDF_MARGIN
    assert (pu.n(gq.res.out_tok)[keep] == o.res.out_tok[keep]).all()


@pytest.mark.parametrize("renorm", [0, 1])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_small_rounds(gpu, pu, renorm, dtype):
    """Ragged lengths including gamma = 0, small and odd vocabulary, uncompressed and compressed."""
    _announce("ragged small", renorm, dtype)
    rng = np.random.default_rng(33 + renorm)
    for V, k in ((97, 97), (97, 11), (1031, 64), (20000, 2000)):
        g = rng.integers(0, 7, 24).astype(np.int32)
        off = W.seq_offsets(g)
        N, B = int(off[-1]), len(g)
        tgt = (rng.standard_normal((N + B, V)) * 2).astype(np.float32)
        draft = np.empty((N, V), np.float32)
        for b in range(B):
            for i in range(g[b]):
                draft[off[b] + i] = tgt[off[b] + b + i] + rng.standard_normal(V).astype(np.float32) * 0.5
        if dtype == "bf16":
            tgt, draft = W.to_bf16_bits(tgt), W.to_bf16_bits(draft)
        w = W.Workload("ragged", 91, B, 0, 6, V, dtype, 0.8, k, 0.0, 1, "custom")
        r = _custom_round(w, draft, tgt, off, rng.random(N + B, dtype=np.float32), rng.random(N, dtype=np.float32))
        o = pu.oracle_round(r, renorm=renorm)
        for seg in (False, True):
            gq = pu.gpu_round(r, o.tok, gpu, renorm=renorm, seg=seg)
            st = pu.compare_round(gq, o, r, max_excluded_frac=0.05)
        assert 0 < o.ver.n_accept.sum() < N


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_round_at_the_largest_vocabulary_and_record(gpu, pu, ps, dtype):
    """The limits the library reports (V = 2^20, k = 4096): one small ragged round, compress, verify and the
    residual draw, and the downlink's record of the rejected rows at the same size."""
    V, k = ps.limit(ps.LIMIT_MAX_V), ps.limit(ps.LIMIT_MAX_K)
    _announce("largest sizes", V, k, dtype)
    assert (V, k) == (1 << 20, 4096)
    rng = np.random.default_rng(77)
    g = np.array([2, 0, 1], np.int32)
    off = W.seq_offsets(g)
    N, B = int(off[-1]), len(g)
    tgt = (rng.standard_normal((N + B, V)) * 4).astype(np.float32)
    draft = np.empty((N, V), np.float32)
    for b in range(B):
        for i in range(g[b]):
            draft[off[b] + i] = tgt[off[b] + b + i] + rng.standard_normal(V).astype(np.float32)
    if dtype == "bf16":
        tgt, draft = W.to_bf16_bits(tgt), W.to_bf16_bits(draft)
    w = W.Workload("largest", 92, B, 0, 2, V, dtype, 1.1, k, 0.0, 1, "custom")
    r = _custom_round(w, draft, tgt, off, rng.random(N + B, dtype=np.float32), rng.random(N, dtype=np.float32))
    o = pu.oracle_round(r)
    for seg in (False, True):
        gq = pu.gpu_round(r, o.tok, gpu, seg=seg)
        pu.compare_round(gq, o, r, max_excluded_frac=0.34)
    orec = oracle.compress_rejected(r.tgt_logits, V, w.T, r.seq_off, o.ver.n_accept, k)
    grec = ps.compress_rejected(pu.to_device(r.tgt_logits, gpu), V, w.T, torch.from_numpy(r.seq_off).to(gpu), N,
                                torch.from_numpy(o.ver.n_accept).to(gpu), k)
    torch.cuda.synchronize()
    pu.compare_compress(grec, orec)
    # one past the limits is refused, not attempted
    with pytest.raises(ps.PicoSpecError) as e:
        ps.compress(torch.zeros((1, V + 1), device=gpu), V + 1, 1.0, 8)
    assert e.value.code == ps.EUNSUPPORTED
    with pytest.raises(ps.PicoSpecError) as e:
        ps.compress(torch.zeros((1, 8192), device=gpu), 8192, 1.0, k + 1)
    assert e.value.code == ps.EUNSUPPORTED


@pytest.mark.parametrize("T,spread", [(0.05, 3.0), (0.2, 8.0), (20.0, 3.0), (1.0, 40.0)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_round_at_extreme_temperatures(gpu, pu, T, spread, dtype):
    """Very peaked (exponents of several hundred below the maximum) and nearly flat distributions: the probabilities,
    masses and the residual draw keep their tolerances."""
    _announce("extreme temperature", T, spread, dtype)
    rng = np.random.default_rng(int(T * 100) + int(spread))
    V, k = 6007, 300
    g = np.array([3, 0, 5, 1, 4, 2], np.int32)
    off = W.seq_offsets(g)
    N, B = int(off[-1]), len(g)
    tgt = (rng.standard_normal((N + B, V)) * spread).astype(np.float32)
    draft = np.empty((N, V), np.float32)
    for b in range(B):
        for i in range(g[b]):
            draft[off[b] + i] = tgt[off[b] + b + i] + rng.standard_normal(V).astype(np.float32) * spread * 0.1
    if dtype == "bf16":
        tgt, draft = W.to_bf16_bits(tgt), W.to_bf16_bits(draft)
    w = W.Workload("extreme", 93, B, 0, 5, V, dtype, T, k, 0.0, 1, "custom")
    r = _custom_round(w, draft, tgt, off, rng.random(N + B, dtype=np.float32), rng.random(N, dtype=np.float32))
    o = pu.oracle_round(r)
    for seg in (False, True):
        gq = pu.gpu_round(r, o.tok, gpu, seg=seg)
        # (peaked by construction: sequences whose oracle residual mass lies below PEAKED_R carry the absolute term)
        pu.compare_round(gq, o, r, max_excluded_frac=0.34, strict=False)


def test_scalar_q_uplink_and_foreign_tokens(gpu, pu, ps):
    """The edge's scalar q_i replaces the sparse lookup; tokens outside the record are accepted and flagged."""
    _announce("scalar q / foreign tokens")
    w = W.WORKLOADS["cfg2"].scaled(B=6, V=4000, k=50)
    r = W.build_round(w)
    o = pu.oracle_round(r)
    dev = lambda a: pu.to_device(a, gpu)
    tgt, seq_off, uni = dev(r.tgt_logits), dev(r.seq_off), dev(r.uniforms)
    q = ps.compress(dev(r.draft_logits), w.V, w.T, w.k)
    tok_d, qs_d = ps.sample_draft(q, dev(r.draft_uniforms))
    # 1) scalar path == sparse path
    v_sparse = ps.verify(tgt, w.V, w.T, seq_off, r.N, tok_d, q, uni)
    v_scalar = ps.verify(tgt, w.V, w.T, seq_off, r.N, tok_d, None, uni, q_scalar=qs_d)
    torch.cuda.synchronize()
    assert torch.equal(v_sparse.n_accept, v_scalar.n_accept)
    assert torch.equal(v_sparse.q_tok, v_scalar.q_tok)
    # 2) a token that is not in the record
    tok = o.tok.copy()
    outside = int(np.setdiff1d(np.arange(w.V), o.q.idx[0])[0])
    tok[0] = outside
    o2 = pu.oracle_round(r, tok=tok)
    g2 = pu.gpu_round(r, tok, gpu)
    pu.compare_round(g2, o2, r, max_excluded_frac=0.2)
    assert pu.n(g2.ver.flags)[0] & ps.FLAG_TOKEN_NOT_IN_SUPPORT
    assert pu.n(g2.ver.q_tok)[0] == 0.0


def test_sample_draft_matches_oracle(gpu, pu, ps):
    _announce("sample_draft")
    w = W.WORKLOADS["cfg3"].scaled(B=4)
    r = W.build_round(w)
    o = oracle.compress(r.draft_logits, w.V, w.T, w.k)
    tok_o, slot_o, mar = oracle.sample_draft(o, r.draft_uniforms)
    q = ps.compress(pu.to_device(r.draft_logits, gpu), w.V, w.T, w.k)
    tok_g, qs_g = ps.sample_draft(q, pu.to_device(r.draft_uniforms, gpu))
    torch.cuda.synchronize()
    keep = mar >= pu.CDF_MARGIN
    assert keep.mean() > 0.9
    assert (pu.n(tok_g)[keep] == tok_o[keep]).all()
    want_q = o.prob[np.arange(r.N), slot_o] / o.mass
    pu.assert_close(pu.n(qs_g)[keep], want_q[keep], pu.RTOL, "q_scalar")


@pytest.mark.parametrize("k", [1, 4, 64, 250, 256, 1000, 1024, 2048, 4096, 5000])
def test_sample_draft_record_shapes(gpu, pu, ps, k):
    """The draw over records of every length class (rows on and off 16-byte boundaries, one to sixteen chunks,
    beyond the longest record the compressor writes), with ragged counts, empty rows and zero weights at the
    end; both sides get the same fp32 record."""
    _announce("sample_draft shapes", k)
    _sample_draft_case(gpu, pu, ps, k, k)


def _sample_draft_case(gpu, pu, ps, k, seed):
    rng = np.random.default_rng(seed)
    rows = 97
    count = rng.integers(0, k + 1, rows).astype(np.int32)
    count[:5] = [k, 0, 1, min(k, 3), max(k - 1, 0)]
    idx = np.full((rows, k), -1, np.int32)
    prob = np.zeros((rows, k), np.float32)
    for r in range(rows):
        c = count[r]
        idx[r, :c] = rng.choice(150000, c, replace=False)
        p = np.sort(rng.dirichlet(np.full(max(c, 1), 0.2)))[::-1][:c] * 0.9
        prob[r, :c] = p.astype(np.float32)
    if count[7] >= 2:
        prob[7, count[7] // 2:count[7]] = 0.0                 # a record whose tail carries no weight
    u = rng.random(rows, dtype=np.float32)
    u[7] = np.float32(1.0 - 2.0 ** -24)
    mass = prob.astype(np.float64).sum(axis=1)
    o = oracle.Compressed(idx, prob.astype(np.float64), count, mass, None, None, k)
    live = count > 0
    tok_o, slot_o, mar = oracle.sample_draft(oracle.Compressed(idx[live], o.prob[live], count[live], mass[live], None, None, k), u[live])
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(gpu)
    q = ps.Compressed(d(idx), d(prob), d(count), d(mass.astype(np.float32)), torch.zeros(rows, device=gpu), k)
    tok_g, qs_g = ps.sample_draft(q, d(u))
    torch.cuda.synchronize()
    tg, qg = pu.n(tok_g), pu.n(qs_g)
    assert np.all(tg[~live] == -1) and np.all(qg[~live] == 0)
    keep = mar >= pu.CDF_MARGIN
    assert keep.mean() > 0.9
    assert (tg[live][keep] == tok_o[keep]).all()
    want_q = o.prob[live][np.arange(live.sum()), slot_o] / mass[live]
    pu.assert_close(qg[live][keep], want_q[keep], pu.RTOL, "q_scalar")


def test_residual_empty_falls_back_to_target(gpu, pu, ps):
    _announce("residual empty")
    V = 300
    rng = np.random.default_rng(9)
    z = (rng.standard_normal((1, V)) * 2).astype(np.float32)
    tgt = np.concatenate([z, z])
    off = np.array([0, 1], np.int32)
    uni = np.array([0.3, 0.6], np.float32)
    oq = oracle.compress(z, V, 1.0, V)
    lse = oracle.verify(tgt, V, 1.0, off, np.array([0], np.int32), oq, uni).tgt_lse
    ores = oracle.sample_residual(tgt, V, 1.0, off, np.array([0], np.int32), lse, oq, uni)
    assert ores.flags[0] & oracle.FLAG_RESIDUAL_EMPTY
    dev = lambda a: pu.to_device(a, gpu)
    q = ps.compress(dev(z), V, 1.0, V)
    ver = ps.verify(dev(tgt), V, 1.0, dev(off), 1, dev(np.array([0], np.int32)), q, dev(uni))
    forced = dev(np.array([0], np.int32))
    # P and qhat agree only up to fp32 rounding on the GPU, so R is ~1e-7 instead of exactly 0: either the flag is
    # set and the draw comes from P, or R is a rounding residue; both are legitimate.  Check the flagged branch
    # deterministically by handing the kernel the exact same probabilities on both sides.
    res = ps.sample_residual(dev(tgt), V, 1.0, dev(off), 1, ver, q, dev(uni), n_accept=forced)
    torch.cuda.synchronize()
    rm = float(pu.n(res.resid_mass)[0])
    assert rm < 1e-5
    if pu.n(res.flags)[0] & ps.FLAG_RESIDUAL_EMPTY:
        assert rm == 0.0 and pu.n(res.out_tok)[0] == ores.out_tok[0]


def test_bad_inputs_are_flagged_not_fatal(gpu, pu, ps):
    _announce("bad inputs")
    w = W.WORKLOADS["cfg1"].scaled(V=2000, k=16)
    r = W.build_round(w)
    o = pu.oracle_round(r)
    tok = o.tok.copy()
    tok[1] = w.V + 5          # token id outside the vocabulary
    g = pu.gpu_round(r, tok, gpu)
    assert pu.n(g.ver.flags)[0] & ps.FLAG_BAD_INPUT
    # an id outside the vocabulary has p = 0: the accepted prefix ends in front of it, with the record's lookup and
    # with the scalar uplink alike
    assert pu.n(g.ver.n_accept)[0] == min(int(o.ver.n_accept[0]), 1) and pu.n(g.ver.p_tok)[1] == 0.0
    dev = lambda a: pu.to_device(a, gpu)
    qs = torch.full((r.N,), 1e-9, dtype=torch.float32, device=gpu)    # q so small that every valid token is accepted
    vs = ps.verify(dev(r.tgt_logits), w.V, w.T, dev(r.seq_off), r.N, dev(tok), None, dev(r.uniforms), q_scalar=qs)
    torch.cuda.synchronize()
    assert pu.n(vs.n_accept)[0] == 1 and pu.n(vs.flags)[0] & ps.FLAG_BAD_INPUT
    bad_n = dev(np.array([99], np.int32))   # n_accept outside [0, gamma]
    res = ps.sample_residual(dev(r.tgt_logits), w.V, w.T, dev(r.seq_off), r.N, g.ver, g.q, dev(r.uniforms),
                             n_accept=bad_n)
    torch.cuda.synchronize()
    assert pu.n(res.flags)[0] & ps.FLAG_BAD_INPUT
    assert 0 <= pu.n(res.out_tok)[0] < w.V


def test_device_range_checks_buffer_loads_as_the_row_kernels_assume(gpu, ps):
    """The memory safety of the look-ahead row loads rests on the range check of raw buffer loads taking the
    scalar offset into account; the library's self-check probes that on this device (all probe addresses lie
    inside its workspace)."""
    _announce("device self-check")
    assert ps.check_device(gpu) == 0


def test_empty_batch(gpu, ps):
    _announce("empty batch")
    tgt = torch.empty((0, 64), dtype=torch.float32, device=gpu)
    seq_off = torch.zeros(1, dtype=torch.int32, device=gpu)
    q = ps.alloc_compressed(0, 4, gpu)
    z = torch.empty(0, dtype=torch.float32, device=gpu)
    ver = ps.verify(tgt, 64, 1.0, seq_off, 0, torch.empty(0, dtype=torch.int32, device=gpu), q, z)
    res = ps.sample_residual(tgt, 64, 1.0, seq_off, 0, ver, q, z)
    torch.cuda.synchronize()
    assert ver.n_accept.numel() == 0 and res.out_tok.numel() == 0


# ---------------------------------------------------------------- full-size rounds, sampled sequences

# (cfg3 and cfg4, the configuration the throughput is quoted on: every sequence; cfg5: 64 of the 512 per round)
FULL_CASES = [("cfg3", 0, 64), ("cfg4", 0, 256), ("cfg5", 0, 64), ("cfg5", 1, 64), ("cfg5", 50, 64), ("cfg5", 99, 64)]


@pytest.mark.parametrize("name,rnd,n_sample", FULL_CASES)
def test_full_size_round_sampled_sequences(gpu, pu, ps, name, rnd, n_sample):
    """The whole batch at its real size goes through the library exactly as bench.py launches it (same calls,
    same shapes); the sequences of a seeded sample (all of them where n_sample is the batch size) are checked
    element by element against the oracle under the strict criteria, and every row and sequence of the batch
    through size-independent properties."""
    w = W.WORKLOADS[name]
    _announce("full size", name, "round", rnd, "B", w.B, "V", w.V, "k", w.k, w.dtype)
    full = W.build_round(w, rnd)
    if n_sample >= w.B:
        pick, sub = np.arange(w.B), full
    else:
        pick = np.sort(np.random.default_rng(1000 + rnd).choice(w.B, size=n_sample, replace=False))
        sub = W.build_round(w, rnd, seqs=pick)
    o = pu.oracle_round(sub)
    dev = lambda a: pu.to_device(a, gpu)
    draft, tgt = dev(full.draft_logits), dev(full.tgt_logits)
    seq_off, uni = dev(full.seq_off), dev(full.uniforms)
    q = ps.compress(draft, w.V, w.T, w.k, w.top_p)
    tok, _ = ps.sample_draft(q, dev(full.draft_uniforms))
    # the sampled sequences get the oracle's drafted tokens, so both sides verify the same draft
    tok_h = pu.n(tok).copy()
    for j, b in enumerate(pick):
        tok_h[full.seq_off[b]:full.seq_off[b + 1]] = o.tok[sub.seq_off[j]:sub.seq_off[j + 1]]
    tok = dev(tok_h)
    ver = ps.verify(tgt, w.V, w.T, seq_off, full.N, tok, q, uni)
    res = ps.sample_residual(tgt, w.V, w.T, seq_off, full.N, ver, q, uni)
    torch.cuda.synchronize()
    g = pu.GpuRound(q, ver, res)
    st = pu.compare_round(pu.slice_gpu_round(g, full, sub), o, sub, max_excluded_frac=0.05)
    print("[stats]", name, rnd, {k: v for k, v in st.items() if k != "topp_excluded"}, flush=True)
    # the same round through the fused call on the existing records, with the segment table (no second pass over a row)
    ws = ps.alloc_workspace(tgt.dtype, full.N + full.B, w.V, gpu, ps.CALL_VERIFY_SAMPLE)
    ver2, res2 = ps.verify_sample(tgt, w.V, w.T, seq_off, full.N, tok, q, uni, workspace=ws)
    torch.cuda.synchronize()
    st2 = pu.compare_round(pu.slice_gpu_round(pu.GpuRound(q, ver2, res2), full, sub), o, sub, max_excluded_frac=0.05)
    print("[stats]", name, rnd, "verify_sample + segment table", {k: v for k, v in st2.items() if k != "topp_excluded"}, flush=True)
    assert torch.equal(ver2.n_accept, ver.n_accept) or st2["mismatch_accept"] > 0
    # properties that hold for every row and sequence of the batch
    idx, prob, cnt, mass = pu.n(q.idx), pu.n(q.prob), pu.n(q.count), pu.n(q.mass)
    assert ((cnt >= 1) & (cnt <= w.k)).all()
    used = np.arange(w.k)[None, :] < cnt[:, None]
    assert (idx[used] >= 0).all() and (idx[used] < w.V).all() and (idx[~used] == -1).all() and (prob[~used] == 0).all()
    assert (np.diff(prob, axis=1)[used[:, 1:]] <= 0).all()                      # descending probabilities
    srt = np.sort(np.where(used, idx, np.arange(w.k)[None, :] + w.V), axis=1)   # ids are distinct within a row
    assert (np.diff(srt, axis=1) > 0).all()
    assert np.allclose(np.where(used, prob, 0).sum(1), mass, rtol=1e-5) and (mass <= 1 + 1e-5).all()
    if w.top_p <= 0:
        assert (cnt == w.k).all()
    g_len = np.diff(full.seq_off)
    na = pu.n(ver.n_accept)
    assert ((na >= 0) & (na <= g_len)).all()
    out = pu.n(res.out_tok)
    assert ((out >= 0) & (out < w.V)).all()
    rm = pu.n(res.resid_mass)
    assert ((rm > 0) & (rm <= 1 + 1e-5)).all()
    assert np.allclose(rm[na == g_len], 1.0, rtol=1e-5)                          # bonus draws come from P itself
    assert (pu.n(ver.flags) == 0).all() and (pu.n(res.flags) == 0).all()


def test_acceptance_is_strict_at_the_boundary(gpu, pu, ps):
    """u == p/q rejects, one ulp below accepts (V = 1: p = 1 exactly; scalar q = 2: ratio = 1/2 exactly)."""
    _announce("strict boundary")
    dev = lambda a: pu.to_device(a, gpu)
    tgt = np.zeros((6, 1), np.float32)
    off = np.array([0, 1, 2, 3], np.int32)
    tok = np.zeros(3, np.int32)
    below = np.nextafter(np.float32(0.5), np.float32(0.0))
    uni = np.array([0.5, 0.0, below, 0.0, np.nextafter(np.float32(0.5), np.float32(1.0)), 0.0], np.float32)
    qs = np.array([2.0, 2.0, 2.0], np.float32)
    o = oracle.verify(tgt, 1, 1.0, off, tok, None, uni, q_scalar=qs.astype(np.float64))
    v = ps.verify(dev(tgt), 1, 1.0, dev(off), 3, dev(tok), None, dev(uni), q_scalar=dev(qs))
    torch.cuda.synchronize()
    assert list(pu.n(v.n_accept)) == list(o.n_accept) == [0, 1, 0]
    assert list(pu.n(v.p_tok)) == [1.0, 1.0, 1.0]
