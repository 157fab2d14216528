"""GPU test of sv_decode_step_static, the entry point for callers that cannot allocate.

It must give what sv_decode_step gives with a caller workspace -- the same kernels on the library's own
per-GPU scratch array -- on two calls in a row, the second on a smaller input (the array keeps what the
first call left behind), and also after other calls have used the GPU.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_17777_amd as sv
from oracle.compare import check_index_sets, out_tolerance

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _inputs(seed, B, Hq, Hkv, D, Nv, Nt, dtype=np.float16):
    rng = np.random.default_rng(seed)
    f = lambda *s: rng.standard_normal(s, dtype=np.float32).astype(dtype)
    return dict(q=f(B, Hq, D), k_vis=f(B, Hkv, Nv, D), v_vis=f(B, Hkv, Nv, D), k_txt=f(B, Hkv, Nt, D), v_txt=f(B, Hkv, Nt, D))


def _both_ways(inp, k, vis_len=None, txt_len=None, with_scores=True):
    d = {n: torch.from_numpy(inp[n]).to(DEV) for n in inp}
    shape = sv.make_shape(d["q"], d["k_vis"], d["k_txt"], k, vis_len=vis_len, txt_len=txt_len)
    assert sv.workspace_bytes(shape) <= sv.STATIC_SCRATCH_BYTES
    res = []
    for static in (False, True):
        buf = sv.DecodeBuffers(shape, DEV, with_scores=with_scores)   # all device memory exists before the call
        buf.idx.fill_(-7); buf.count.fill_(-7); buf.out.fill_(float("nan")); buf.lse.fill_(float("nan"))
        torch.cuda.synchronize()
        args = (shape, d["q"], d["k_vis"], d["v_vis"], d["k_txt"], d["v_txt"], buf.scores, buf.idx, buf.count, buf.out, buf.lse)
        if static:
            sv.sv_decode_step_static(*args)
        else:
            sv.sv_decode_step(*args, buf.workspace)
        torch.cuda.synchronize()
        res.append(dict(scores=None if buf.scores is None else buf.scores.cpu().numpy(), idx=buf.idx.cpu().numpy(),
                        count=buf.count.cpu().numpy(), out=buf.out.cpu().numpy(), lse=buf.lse.cpu().numpy()))
    return res


def _assert_same(ws, st, inp, k, vis_len, txt_len, label):
    # integer outputs bit for bit; floating-point outputs to the bar of the parity tests (the two calls run the
    # same kernels in the same launch shapes, so they are expected to agree to the bit, which is also checked)
    assert np.array_equal(st["idx"], ws["idx"]) and np.array_equal(st["count"], ws["count"]), label
    tol = out_tolerance(inp["q"].dtype)
    assert np.all(np.isfinite(st["out"])), label
    assert np.abs(st["out"] - ws["out"]).max() <= tol, label
    fin = np.isfinite(ws["lse"])
    assert np.array_equal(np.isfinite(st["lse"]), fin) and np.abs(st["lse"] - ws["lse"])[fin].max(initial=0.0) <= tol, label
    assert np.array_equal(st["out"], ws["out"]) and np.array_equal(st["lse"], ws["lse"]), f"{label}: not bit-identical"
    if ws["scores"] is not None:
        assert np.array_equal(st["scores"], ws["scores"]), label
    # and against the oracle, so that two equal wrong answers cannot pass
    o = oracle.decode_step(inp["q"], inp["k_vis"], inp["v_vis"], inp["k_txt"], inp["v_txt"], k, vis_len=vis_len, txt_len=txt_len)
    assert check_index_sets(o["scores"], k, vis_len, st["idx"], st["count"]).ok, label
    oa, _, _ = oracle.sparse_decode_attn(inp["q"], inp["k_vis"], inp["v_vis"], inp["k_txt"], inp["v_txt"], st["idx"], st["count"],
                                         txt_len=txt_len)
    assert np.abs(st["out"] - oa).max() <= tol, label


def test_static_scratch_step_equals_the_workspace_step_on_two_calls_the_second_smaller():
    # first call: long rows (candidate filter, records and threshold words in the scratch array), ragged batch
    big = _inputs(5101, 3, 28, 4, 128, 20000, 700)
    vis_len, txt_len = np.array([20000, 17011, 18500], np.int32), np.array([700, 1, 333], np.int32)
    ws, st = _both_ways(big, 1000, vis_len, txt_len, with_scores=False)
    _assert_same(ws, st, big, 1000, vis_len, txt_len, "first, long rows")
    # second call, smaller in every dimension: short rows (scores in the scratch array, one workgroup per row selects)
    small = _inputs(5102, 2, 8, 2, 128, 3000, 90)
    ws, st = _both_ways(small, 300, None, None, with_scores=False)
    _assert_same(ws, st, small, 300, None, None, "second, smaller")
    # third: fp32 / head_dim 64 with a scores buffer of the caller's, after the two above
    tiny = _inputs(5103, 1, 4, 1, 64, 512, 64, np.float32)
    ws, st = _both_ways(tiny, 64, None, None, with_scores=True)
    _assert_same(ws, st, tiny, 64, None, None, "third, fp32")


def test_static_scratch_step_rejects_a_shape_beyond_its_array():
    q = torch.zeros((28, 28, 128), dtype=torch.float16, device=DEV)
    k_vis = torch.empty((28, 4, 50176, 128), dtype=torch.float16, device=DEV)
    k_txt = torch.empty((28, 4, 1024, 128), dtype=torch.float16, device=DEV)
    shape = sv.make_shape(q, k_vis, k_txt, 2509)
    assert sv.workspace_bytes(shape) > sv.STATIC_SCRATCH_BYTES
    idx = torch.empty((28, 4, 2509), dtype=torch.int32, device=DEV)
    cnt = torch.empty((28, 4), dtype=torch.int32, device=DEV)
    out = torch.full((28, 28, 128), 3.0, dtype=torch.float32, device=DEV)
    with pytest.raises(sv.SVError) as e:
        sv.sv_decode_step_static(shape, q, k_vis, k_vis, k_txt, k_txt, None, idx, cnt, out, None)
    assert e.value.status == -5
    torch.cuda.synchronize()
    assert bool((out == 3.0).all())       # nothing was launched
