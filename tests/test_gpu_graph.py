"""The library's calls only enqueue kernels on the caller's stream, so a round can be captured into a
HIP graph.  The captured round is replayed several times, with eager work and synchronisation between
the replays, and every replay must reproduce the eager results bit for bit."""
import numpy as np
import pytest
import torch

from paper_2603_19133_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_captured_round_replays_identically(gpu):
    import parity_util as pu
    from paper_2603_19133_amd import binding as ps
    print("[case] graph capture of a round", flush=True)
    w = W.WORKLOADS["cfg3"].scaled(B=6)
    r = W.build_round(w, 0)
    draft, tgt = pu.to_device(r.draft_logits, gpu), pu.to_device(r.tgt_logits, gpu)
    seq_off = torch.from_numpy(r.seq_off).to(gpu)
    uni, duni = torch.from_numpy(r.uniforms).to(gpu), torch.from_numpy(r.draft_uniforms).to(gpu)
    q = ps.alloc_compressed(r.N, w.k, gpu)
    ver = ps.alloc_verified(r.B, r.N, gpu)
    res = ps.alloc_residual(r.B, gpu)
    ps.compress(draft, w.V, w.T, w.k, w.top_p, out=q)
    tok, _ = ps.sample_draft(q, duni)

    def round_():
        ps.compress(draft, w.V, w.T, w.k, w.top_p, out=q)
        ps.verify(tgt, w.V, w.T, seq_off, r.N, tok, q, uni, out=ver)
        ps.sample_residual(tgt, w.V, w.T, seq_off, r.N, ver, q, uni, out=res)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (q.idx, q.prob, q.count, q.mass, q.lse, ver.n_accept, ver.p_tok, ver.q_tok,
                                    ver.tgt_max, ver.tgt_sum, ver.flags, res.out_tok, res.resid_mass, res.flags)]

    round_()                                   # eager (also sets the kernels' attributes before the capture)
    want = snapshot()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            round_()
    for rep in range(3):
        for t in (q.idx, q.prob, ver.n_accept, res.out_tok):      # eager work between the replays: spoil the outputs
            t.fill_(-7)
        torch.cuda.synchronize()
        g.replay()
        got = snapshot()
        for a, b in zip(got, want):
            assert torch.equal(a, b), f"replay {rep} differs"
