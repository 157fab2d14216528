"""Helpers for the GPU parity tests: numpy inputs -> device tensors -> C-ABI calls -> numpy."""
from __future__ import annotations

import numpy as np
import torch

import paper_2510_17777_amd as sv

DEV = "cuda:0"


def to_dev(inp: dict) -> dict:
    d = {}
    for key in ("q", "k_vis", "v_vis", "k_txt", "v_txt"):
        d[key] = torch.from_numpy(np.ascontiguousarray(inp[key])).to(DEV)
    return d


def run_step(inp: dict, k: int, vis_len=None, txt_len=None, scale: float = 0.0, dev=None,
             with_scores: bool = True) -> dict:
    """sv_decode_step through the C ABI; returns numpy scores/idx/count/out/lse."""
    d = dev if dev is not None else to_dev(inp)
    shape = sv.make_shape(d["q"], d["k_vis"], d["k_txt"], k, vis_len=vis_len, txt_len=txt_len, scale=scale)
    buf = sv.DecodeBuffers(shape, DEV, with_scores=with_scores)
    if k > 0:
        buf.idx.fill_(-7)
    buf.count.fill_(-7)
    buf.out.fill_(float("nan"))
    sv.sv_decode_step(shape, d["q"], d["k_vis"], d["v_vis"], d["k_txt"], d["v_txt"],
                      buf.scores, buf.idx, buf.count, buf.out, buf.lse, buf.workspace)
    torch.cuda.synchronize()
    return dict(scores=None if buf.scores is None else buf.scores.cpu().numpy(),
                idx=buf.idx.cpu().numpy(), count=buf.count.cpu().numpy(),
                out=buf.out.cpu().numpy(), lse=buf.lse.cpu().numpy(), shape=shape, buf=buf, dev=d)


def run_stages(inp: dict, k: int, vis_len=None, txt_len=None, scale: float = 0.0, idx=None, count=None) -> dict:
    """The three entry points one by one; idx/count (numpy) may be supplied for step 3."""
    d = to_dev(inp)
    shape = sv.make_shape(d["q"], d["k_vis"], d["k_txt"], k, vis_len=vis_len, txt_len=txt_len, scale=scale)
    buf = sv.DecodeBuffers(shape, DEV)
    sv.sv_score_visual(shape, d["q"], d["k_vis"], buf.scores)
    sv.sv_topk_select(shape, buf.scores, buf.idx, buf.count, buf.workspace)
    torch.cuda.synchronize()
    sel_idx, sel_count = buf.idx.cpu().numpy(), buf.count.cpu().numpy()
    if idx is not None:
        buf.idx.copy_(torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int32)))
        buf.count.copy_(torch.from_numpy(np.ascontiguousarray(count, dtype=np.int32)))
    sv.sv_sparse_decode_attn(shape, d["q"], d["k_vis"], d["v_vis"], d["k_txt"], d["v_txt"],
                             buf.idx, buf.count, buf.out, buf.lse, buf.workspace)
    torch.cuda.synchronize()
    return dict(scores=buf.scores.cpu().numpy(), idx=sel_idx, count=sel_count,
                out=buf.out.cpu().numpy(), lse=buf.lse.cpu().numpy())


def score_error_bound(inp: dict, scale: float) -> np.ndarray:
    """Per-element bound on |fp32 score - exact score|.

    The kernel adds the G query rows in fp32 (relative error <= (G-1)u per component),
    accumulates D products in fp32 (<= (D+1)u relative to sum |q_d K_d|), and scales once:
    bound = (G + D + 2) * u * scale * sum_d |qsum_d| |K_jd|, u = 2^-24, doubled for slack.
    """
    q = inp["q"].astype(np.float64)
    K = inp["k_vis"].astype(np.float64)
    B, Hq, D = q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    qabs = np.abs(q.reshape(B, Hkv, G, D)).sum(axis=2)
    mag = np.einsum("bgd,bgnd->bgn", qabs, np.abs(K))
    return 2.0 * (G + D + 2) * 2.0 ** -24 * scale * mag + 1e-30
