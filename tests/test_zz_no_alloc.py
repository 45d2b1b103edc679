"""picospec_verify_sample_static (the entry point that allocates nothing: its scratch is a fixed array in the
library's device image) against picospec_verify_sample, through the C ABI: two calls in a row on one stream, the
second with a smaller input, every output equal bit for bit (same kernels), and the round equal to the oracle's."""
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


def _inputs(pu, ps, gpu, w, rnd):
    r = W.build_round(w, rnd)
    o = pu.oracle_round(r)
    d = lambda a: pu.to_device(a, gpu)
    tgt, seq_off, uni, tok = d(r.tgt_logits), d(r.seq_off), d(r.uniforms), d(o.tok)
    q = ps.compress(d(r.draft_logits), w.V, w.T, w.k, w.top_p)
    return r, o, tgt, seq_off, uni, tok, q


def test_no_alloc_entry_point_matches_verify_sample(gpu, pu, ps):
    print("[case] verify_sample_static, two calls in a row", flush=True)
    big = W.WORKLOADS["cfg5"].scaled(B=40)                    # ragged, bf16, top-p records
    small = W.WORKLOADS["cfg3"].scaled(B=5)                   # fewer and shorter rows: the array keeps the first call's table
    cases = []
    for w, rnd in ((big, 3), (small, 0)):
        r, o, tgt, seq_off, uni, tok, q = _inputs(pu, ps, gpu, w, rnd)
        ver = ps.alloc_verified(r.B, r.N, gpu)
        res = ps.alloc_residual(r.B, gpu)
        cases.append((w, r, o, tgt, seq_off, uni, tok, q, ver, res))
    # (a first call, so that the runtime has loaded the kernels and the device image before memory is looked at)
    w, r, o, tgt, seq_off, uni, tok, q, ver, res = cases[1]
    ps.verify_sample_static(tgt, w.V, w.T, seq_off, r.N, tok, q, uni, ver, res)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    for w, r, o, tgt, seq_off, uni, tok, q, ver, res in cases:           # back to back on one stream
        ps.verify_sample_static(tgt, w.V, w.T, seq_off, r.N, tok, q, uni, ver, res)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before                   # nothing was allocated on the device
    for w, r, o, tgt, seq_off, uni, tok, q, ver, res in cases:
        ws = ps.alloc_workspace(tgt.dtype, r.N + r.B, w.V, gpu, ps.CALL_VERIFY_SAMPLE)
        ver2, res2 = ps.verify_sample(tgt, w.V, w.T, seq_off, r.N, tok, q, uni, workspace=ws)
        torch.cuda.synchronize()
        for a, b in ((ver.n_accept, ver2.n_accept), (ver.p_tok, ver2.p_tok), (ver.q_tok, ver2.q_tok), (ver.tgt_max, ver2.tgt_max),
                     (ver.tgt_sum, ver2.tgt_sum), (ver.tgt_lse, ver2.tgt_lse), (ver.flags, ver2.flags),
                     (res.out_tok, res2.out_tok), (res.resid_mass, res2.resid_mass), (res.flags, res2.flags)):
            assert torch.equal(a, b)
        pu.compare_round(pu.GpuRound(q, ver, res), o, r, max_excluded_frac=0.2)


def test_no_alloc_entry_point_rejects_what_does_not_fit(gpu, ps):
    print("[case] verify_sample_static, table beyond the fixed array", flush=True)
    assert ps.static_scratch_bytes() == 8 << 20
    V, rows = 1 << 20, 4096                                   # 4096 rows of 2^20 fp32 elements: a table of 33 MB
    assert ps.workspace_bytes(ps.CALL_VERIFY_SAMPLE, ps.F32, rows, V, 8) > ps.static_scratch_bytes()
    fake = 0x1000                                             # (the call fails its size check before anything is touched)
    rc = ps.lib.picospec_verify_sample_static(fake, ps.F32, V, V, 1.0, 1, rows - 1, fake, fake, fake, fake, fake, fake, 8, 1, fake,
                                              fake, fake, fake, fake, fake, fake, fake, fake, fake, fake, None)
    assert rc == ps.ESCRATCH
    assert b"picospec_verify_sample_static" in ps.lib.picospec_strerror(rc)
