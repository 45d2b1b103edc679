"""A round recorded into a HIP graph (a serving loop replays it without launching from the host): every replay,
with fresh inputs copied into the same buffers and eager work in between, gives bit for bit what the eager
call gives on those inputs.  The eager call itself is checked against the oracle elsewhere."""
import numpy as np
import pytest
import torch

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


def _fields(q, ver, res):
    return dict(idx=q.idx, prob=q.prob, count=q.count, mass=q.mass, lse=q.lse, n_accept=ver.n_accept, p_tok=ver.p_tok,
                q_tok=ver.q_tok, tgt_max=ver.tgt_max, tgt_sum=ver.tgt_sum, tgt_lse=ver.tgt_lse, vflags=ver.flags,
                out_tok=res.out_tok, resid_mass=res.resid_mass, rflags=res.flags)


# (two launches: 64 + 72 rows), (three launches: 320 + 360 rows), fp32 rows with the separate calls recorded
@pytest.mark.parametrize("name,scale,one_call", [("cfg2", {}, True), ("cfg3", {"B": 40}, True), ("cfg4", {"B": 6}, False)])
def test_graph_replays_match_eager(gpu, ps, pu, name, scale, one_call):
    print("[case] graph", name, scale, one_call, flush=True)
    w = W.WORKLOADS[name].scaled(**scale) if scale else W.WORKLOADS[name]
    rounds = [W.build_round(w, i) for i in range(3)]
    r0 = rounds[0]
    assert all(np.array_equal(r.seq_off, r0.seq_off) for r in rounds)      # fixed gamma: the same shape every round
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(gpu)
    seq_off = d(r0.seq_off)

    def call(draft, tgt, tok, uni, q, ver, res):
        if one_call:
            ps.round(draft, tgt, w.V, w.T, seq_off, r0.N, tok, w.k, uni, top_p=w.top_p, q=q, ver=ver, res=res)
        else:
            ps.compress(draft, w.V, w.T, w.k, w.top_p, out=q)
            ps.verify(tgt, w.V, w.T, seq_off, r0.N, tok, q, uni, out=ver)
            ps.sample_residual(tgt, w.V, w.T, seq_off, r0.N, ver, q, uni, out=res)

    # eager results of every round, each into buffers of its own
    inputs, eager = [], []
    for r in rounds:
        draft, tgt, uni = pu.to_device(r.draft_logits, gpu), pu.to_device(r.tgt_logits, gpu), d(r.uniforms)
        q = ps.compress(draft, w.V, w.T, w.k, w.top_p)
        tok, _ = ps.sample_draft(q, d(r.draft_uniforms))
        q, ver, res = ps.alloc_compressed(r.N, w.k, gpu), ps.alloc_verified(r.B, r.N, gpu), ps.alloc_residual(r.B, gpu)
        call(draft, tgt, tok, uni, q, ver, res)
        torch.cuda.synchronize()
        inputs.append((draft, tgt, tok, uni))
        eager.append({k: v.clone() for k, v in _fields(q, ver, res).items()})

    # the graph works on static buffers
    s_in = [t.clone() for t in inputs[0]]
    q, ver, res = ps.alloc_compressed(r0.N, w.k, gpu), ps.alloc_verified(r0.B, r0.N, gpu), ps.alloc_residual(r0.B, gpu)
    out = _fields(q, ver, res)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call(*s_in, q, ver, res)
    for i in (1, 2, 0, 2):
        for dst, src in zip(s_in, inputs[i]):
            dst.copy_(src)
        for v in out.values():                       # whatever a replay does not write would show
            v.fill_(-3)
        g.replay()
        torch.cuda.synchronize()
        for k, v in out.items():
            assert torch.equal(v, eager[i][k]), (i, k)
        scratch = torch.randn(1 << 16, device=gpu).sum().item()           # eager work between the replays
        assert np.isfinite(scratch)


def test_calls_on_two_streams_do_not_disturb_each_other(gpu, ps, pu):
    """The library keeps no mutable state between calls: two rounds enqueued on two streams at the same time give
    what each gives alone."""
    print("[case] two streams", flush=True)
    ws = [W.WORKLOADS["cfg3"].scaled(B=24), W.WORKLOADS["cfg4"].scaled(B=10)]
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(gpu)
    jobs = []
    for w in ws:
        r = W.build_round(w, 0)
        draft, tgt = pu.to_device(r.draft_logits, gpu), pu.to_device(r.tgt_logits, gpu)
        q = ps.compress(draft, w.V, w.T, w.k, w.top_p)
        tok, _ = ps.sample_draft(q, d(r.draft_uniforms))
        args = (draft, tgt, w.V, w.T, d(r.seq_off), r.N, tok, w.k, d(r.uniforms))
        alone = ps.round(*args, top_p=w.top_p)
        torch.cuda.synchronize()
        jobs.append((args, w, {k: v.clone() for k, v in _fields(*alone).items()}))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(5):
        outs = []
        for (args, w, _), s in zip(jobs, streams):
            s.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(s):
                outs.append(ps.round(*args, top_p=w.top_p))
        torch.cuda.synchronize()
        for (args, w, want), got in zip(jobs, outs):
            for k, v in _fields(*got).items():
                assert torch.equal(v, want[k]), (rep, w.name, k)
