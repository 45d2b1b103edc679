"""The seeded input generators: determinism, layout, and the stated recipes (CPU only)."""
import numpy as np
import pytest

from paper_2603_19133_amd import workloads as W


def test_five_workloads_have_the_stated_shapes():
    w = W.WORKLOADS
    assert (w["cfg1"].B, w["cfg1"].gamma_hi, w["cfg1"].V, w["cfg1"].dtype, w["cfg1"].k) == (1, 4, 32000, "f32", 64)
    assert (w["cfg2"].B, w["cfg2"].gamma_hi, w["cfg2"].V, w["cfg2"].dtype, w["cfg2"].k) == (8, 8, 32000, "bf16", 256)
    assert (w["cfg3"].B, w["cfg3"].V, w["cfg3"].T, w["cfg3"].k) == (64, 128256, 0.7, 1024)
    assert (w["cfg4"].B, w["cfg4"].gamma_hi, w["cfg4"].V, w["cfg4"].dtype, w["cfg4"].k) == (256, 16, 151936, "f32", 4096)
    assert (w["cfg5"].B, w["cfg5"].gamma_lo, w["cfg5"].gamma_hi, w["cfg5"].V, w["cfg5"].top_p, w["cfg5"].k,
            w["cfg5"].rounds) == (512, 1, 16, 152064, 0.95, 2048, 100)


def test_round_layout_and_determinism():
    w = W.WORKLOADS["cfg2"].scaled(V=1000)
    a, b = W.build_round(w), W.build_round(w, workers=1)
    assert a.draft_logits.shape == (64, 1000) and a.tgt_logits.shape == (72, 1000)
    assert a.draft_logits.dtype == np.uint16
    assert (a.draft_logits == b.draft_logits).all() and (a.tgt_logits == b.tgt_logits).all()
    assert (a.uniforms == b.uniforms).all() and a.uniforms.dtype == np.float32
    assert a.uniforms.min() >= 0 and a.uniforms.max() < 1
    assert list(a.seq_off) == list(range(0, 65, 8))


def test_subset_of_sequences_equals_full_batch():
    w = W.WORKLOADS["cfg5"].scaled(B=12, V=500)
    full = W.build_round(w, rnd=3)
    sub = W.build_round(w, rnd=3, seqs=[2, 7, 11])
    g = W.gammas(w, 3)
    assert 1 <= g.min() and g.max() <= 16 and len(set(g.tolist())) > 1
    for j, b in enumerate([2, 7, 11]):
        fo, so = full.seq_off, sub.seq_off
        assert (sub.draft_logits[so[j]:so[j + 1]] == full.draft_logits[fo[b]:fo[b + 1]]).all()
        assert (sub.tgt_logits[so[j] + j:so[j + 1] + j + 1] == full.tgt_logits[fo[b] + b:fo[b + 1] + b + 1]).all()
        assert (sub.uniforms[so[j] + j:so[j + 1] + j + 1] == full.uniforms[fo[b] + b:fo[b + 1] + b + 1]).all()
        assert (sub.draft_uniforms[so[j]:so[j + 1]] == full.draft_uniforms[fo[b]:fo[b + 1]]).all()
    other = W.build_round(w, rnd=4)
    assert not np.array_equal(W.gammas(w, 4), g)
    # logits are fixed across rounds per (sequence, position); only lengths and uniforms change
    b = 0
    n = min(g[b], W.gammas(w, 4)[b])
    assert (other.tgt_logits[other.seq_off[b] + b][:] == full.tgt_logits[full.seq_off[b] + b]).all() and n >= 1


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.005859375, 1.01171875, -2.5, 3.0e38], np.float32)
    bits = W.to_bf16_bits(x)
    back = W.bf16_bits_to_f32(bits)
    assert back[0] == 1.0
    assert back[1] == 1.0            # 1 + 2^-8 is a tie between 1 and 1+2^-7 -> even mantissa (1.0)
    assert back[2] == 1.0078125      # above the tie -> up
    assert back[3] == 1.015625       # 1 + 3*2^-8 is a tie -> even mantissa (1 + 2^-6)
    assert back[4] == -2.5
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)


@pytest.mark.parametrize("name,std", [("cfg1", 3.0), ("cfg2", 4.0), ("cfg4", 5.0)])
def test_normal_recipes_have_the_stated_scale(name, std):
    w = W.WORKLOADS[name]
    t = W.target_row(w, 0, 0)
    assert abs(t.std() - std) / std < 0.02 and abs(t.mean()) < 0.1
    d = W.draft_row(w, 0, 0, t)
    if name == "cfg1":
        assert abs((d - t).std() - 1.0) < 0.02
    if name == "cfg2":
        assert abs((d - np.float32(0.8) * t).std() - 1.5) < 0.03
    if name == "cfg4":
        frac = (d != t).mean()
        assert abs(frac - 0.1) < 0.005
        assert abs(d[d != t].std() - 5.0) < 0.2


@pytest.mark.parametrize("name,s", [("cfg3", 1.1), ("cfg5", 1.2)])
def test_zipf_recipe_shape(name, s):
    w = W.WORKLOADS[name]
    t = W.target_row(w, 1, 2)
    assert t.shape == (w.V,)
    srt = np.sort(t)[::-1]
    # the sorted profile follows -s*ln(rank) up to the 0.5-sigma jitter
    ranks = np.array([10, 100, 1000, 10000])
    assert np.allclose(srt[ranks - 1], -s * np.log(ranks), atol=1.5)
    assert t.max() < 3.0 and t.min() < -s * np.log(w.V) + 1.0
