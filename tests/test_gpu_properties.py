"""Properties of the GPU path that hold at any size and need no oracle: the token a round emits first follows the
target distribution exactly when the draft token was drawn from the renormalised record the test is run with
(the losslessness the rule of Section 3.3 is built for), whatever the record's length."""
import numpy as np
import pytest
import scipy.stats
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ps():
    from paper_2603_19133_amd import binding
    return binding


def _softmax64(z, T):
    z = z.astype(np.float64) / T
    e = np.exp(z - z.max())
    return e / e.sum()


@pytest.mark.parametrize("V,k,dtype,T,one_call", [(8, 8, torch.float32, 1.0, False), (8, 3, torch.float32, 1.0, True),
                                                  (8, 5, torch.bfloat16, 0.7, True), (300, 32, torch.bfloat16, 1.3, False),
                                                  (5000, 64, torch.float32, 1.0, True)])
def test_first_emitted_token_follows_the_target_distribution(gpu, ps, V, k, dtype, T, one_call):
    print("[case] emitted-token distribution", V, k, dtype, T, one_call, flush=True)
    n = 200_000 if V <= 300 else 60_000
    rng = np.random.default_rng(7 * V + k)
    zt = (rng.standard_normal(V) * 1.5).astype(np.float32)
    zd = (zt + rng.standard_normal(V).astype(np.float32)).astype(np.float32)
    zt_d, zd_d = torch.from_numpy(zt).to(gpu).to(dtype), torch.from_numpy(zd).to(gpu).to(dtype)
    p = _softmax64(zt_d.float().cpu().numpy(), T)                       # the distribution of the logits as stored
    tgt = zt_d.repeat(2 * n, 1)
    draft = zd_d.repeat(n, 1)
    off = torch.arange(n + 1, dtype=torch.int32, device=gpu)            # gamma = 1 everywhere
    g = torch.Generator(device=gpu)
    g.manual_seed(V + k)
    uni = torch.rand(2 * n, device=gpu, generator=g)
    q = ps.compress(draft, V, T, k)
    tok, _ = ps.sample_draft(q, torch.rand(n, device=gpu, generator=g))
    if one_call:
        _, ver, res = ps.round(draft, tgt, V, T, off, n, tok, k, uni)
    else:
        ver = ps.verify(tgt, V, T, off, n, tok, q, uni)
        res = ps.sample_residual(tgt, V, T, off, n, ver, q, uni)
    torch.cuda.synchronize()
    assert int(ver.flags.max().item()) == 0 and int(res.flags.max().item()) == 0
    emitted = torch.where(ver.n_accept == 1, tok, res.out_tok).cpu().numpy()
    obs = np.bincount(emitted, minlength=V).astype(np.float64)
    exp = p * n
    # pool the tail so that every cell expects at least 20 draws
    order = np.argsort(-exp)
    keep = order[exp[order] >= 20]
    o = np.append(obs[keep], obs.sum() - obs[keep].sum())
    e = np.append(exp[keep], exp.sum() - exp[keep].sum())
    if e[-1] < 20:
        o, e = np.append(o[:-2], o[-2:].sum()), np.append(e[:-2], e[-2:].sum())
    chi = scipy.stats.chisquare(o, e)
    assert chi.pvalue > 1e-3, (chi, len(o))
    # and the acceptance rate is sum_x min(P(x), qhat(x)) with qhat the renormalised record
    qd = _softmax64(zd_d.float().cpu().numpy(), T)
    top = np.lexsort((np.arange(V), -zd_d.float().cpu().numpy().astype(np.float64)))[:k]
    qh = np.zeros(V)
    qh[top] = qd[top] / qd[top].sum()
    alpha = np.minimum(p, qh).sum()
    rate = float((ver.n_accept == 1).float().mean().item())
    assert abs(rate - alpha) < 5 * np.sqrt(alpha * (1 - alpha) / n) + 1e-6, (rate, alpha)


def test_unrenormalised_truncated_record_is_detectably_biased(gpu, ps):
    """The check above has the power to see a wrong qhat: with k < V and the record's raw values (renorm 0) the
    test runs with a q the token was not drawn from, and the emitted distribution is off."""
    print("[case] emitted-token distribution, negative control", flush=True)
    V, k, n = 8, 3, 200_000
    rng = np.random.default_rng(103)
    zt = (rng.standard_normal(V) * 1.5).astype(np.float32)
    zd = (zt + rng.standard_normal(V).astype(np.float32)).astype(np.float32)
    tgt = torch.from_numpy(zt).to(gpu).repeat(2 * n, 1)
    draft = torch.from_numpy(zd).to(gpu).repeat(n, 1)
    off = torch.arange(n + 1, dtype=torch.int32, device=gpu)
    g = torch.Generator(device=gpu)
    g.manual_seed(5)
    uni = torch.rand(2 * n, device=gpu, generator=g)
    q = ps.compress(draft, V, 1.0, k)
    tok, _ = ps.sample_draft(q, torch.rand(n, device=gpu, generator=g))
    _, ver, res = ps.round(draft, tgt, V, 1.0, off, n, tok, k, uni, renorm=0)
    torch.cuda.synchronize()
    emitted = torch.where(ver.n_accept == 1, tok, res.out_tok).cpu().numpy()
    obs = np.bincount(emitted, minlength=V)
    assert scipy.stats.chisquare(obs, _softmax64(zt, 1.0) * n).pvalue < 1e-6
