"""CPU oracle of the sparse decode step -- TEST INFRASTRUCTURE, not product code.

Thin ctypes access to ``sv_oracle.c`` (plain C, double precision; the three
steps of the paper's section 3.2 written out as their definitions).  Only
``tests/``, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package; the HIP library and its Python binding never do, and
this package imports nothing from them.

Arrays are numpy, contiguous, ``[B, Hkv, N, D]`` for K/V and ``[B, Hq, D]``
for q; dtype float16 or float32 decides how the C code widens the bits.

Three further definitions are written out here in numpy float64 with the
attention matrix formed explicitly: ``pack_selected`` (section 3.2, packing),
``score_visual_mass`` (section 3.2, retrieval with a multi-token question)
and ``salience_self`` (section 3.1, query-agnostic salience of an encoder
layer).  Every function is pinned in ``tests/test_oracle_pins.py``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sv_oracle.c")
_LIB = os.path.join(_HERE, "libsv_oracle.so")
_lib: Optional[ctypes.CDLL] = None


# SV_ORACLE_SANITIZE=1: the same source built with AddressSanitizer and UndefinedBehaviorSanitizer into a library of
# its own (the process must then run with gcc's libasan preloaded; see tests/run_sanitizers.sh).
_SANITIZE = os.environ.get("SV_ORACLE_SANITIZE", "0") not in ("", "0")
if _SANITIZE:
    _LIB = os.path.join(_HERE, "libsv_oracle_asan.so")


def build(force: bool = False) -> str:
    """Compile sv_oracle.c with gcc (OpenMP over independent (batch, head) units)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        opt = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
               "-fno-sanitize-recover=undefined"] if _SANITIZE else ["-O2"]
        cmd = ["gcc", *opt, "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, ip, dp = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
        i, d = ctypes.c_int, ctypes.c_double
        lib.svo_half_to_double.restype = ctypes.c_double
        lib.svo_half_to_double.argtypes = [ctypes.c_uint16]
        lib.svo_score_visual.restype = i
        lib.svo_score_visual.argtypes = [i, i, i, i, i, i, d, vp, vp, ip, dp]
        lib.svo_topk_select.restype = i
        lib.svo_topk_select.argtypes = [i, i, i, i, dp, ip, ip, ip]
        lib.svo_sparse_decode_attn.restype = i
        lib.svo_sparse_decode_attn.argtypes = [i, i, i, i, i, i, i, i, d, vp, vp, vp, vp, vp,
                                               ip, ip, ip, dp, dp, dp]
        lib.svo_decode_step.restype = i
        lib.svo_decode_step.argtypes = [i, i, i, i, i, i, i, i, d, vp, vp, vp, vp, vp,
                                        ip, ip, dp, ip, ip, dp, dp, dp]
        _lib = lib
    return _lib


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float16:
        return 0
    if a.dtype == np.float32:
        return 1
    raise TypeError(f"oracle inputs must be float16 or float32, got {a.dtype}")


def _c(a: np.ndarray, dtype=None) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _lens(x, B: int) -> Optional[np.ndarray]:
    if x is None:
        return None
    x = np.ascontiguousarray(x, dtype=np.int32)
    assert x.shape == (B,)
    return x


def half_to_double(bits: int) -> float:
    return float(_load().svo_half_to_double(int(bits)))


def default_scale(D: int) -> float:
    return 1.0 / float(np.sqrt(np.float64(D)))


def score_visual(q, k_vis, vis_len=None, scale: Optional[float] = None) -> np.ndarray:
    """Step 1: float64 scores [B, Hkv, Nv]; -inf beyond vis_len."""
    q, k_vis = _c(q), _c(k_vis)
    B, Hq, D = q.shape
    _, Hkv, Nv, _ = k_vis.shape
    assert k_vis.shape == (B, Hkv, Nv, D) and q.dtype == k_vis.dtype
    vl = _lens(vis_len, B)
    s = np.empty((B, Hkv, Nv), dtype=np.float64)
    rc = _load().svo_score_visual(B, Hq, Hkv, D, Nv, _dtype_code(q),
                                  default_scale(D) if scale is None else scale,
                                  _ptr(q), _ptr(k_vis), _ptr(vl), _ptr(s))
    if rc:
        raise ValueError(f"svo_score_visual failed: {rc}")
    return s


def topk_select(scores, k: int, vis_len=None):
    """Step 2: (idx [B,Hkv,k] int32 ascending, -1 padded; count [B,Hkv] int32)."""
    s = _c(scores, np.float64)
    B, Hkv, Nv = s.shape
    vl = _lens(vis_len, B)
    idx = np.full((B, Hkv, max(k, 0)), -1, dtype=np.int32)
    cnt = np.zeros((B, Hkv), dtype=np.int32)
    rc = _load().svo_topk_select(B, Hkv, Nv, k, _ptr(s), _ptr(vl), _ptr(idx), _ptr(cnt))
    if rc:
        raise ValueError(f"svo_topk_select failed: {rc}")
    return idx, cnt


def sparse_decode_attn(q, k_vis, v_vis, k_txt, v_txt, idx, count, txt_len=None,
                       scale: Optional[float] = None):
    """Step 3: (out [B,Hq,D] f64, lse [B,Hq] f64, wsum [B,Hq] f64)."""
    q, k_vis, v_vis, k_txt, v_txt = map(_c, (q, k_vis, v_vis, k_txt, v_txt))
    B, Hq, D = q.shape
    _, Hkv, Nv, _ = k_vis.shape
    Nt = k_txt.shape[2]
    assert v_vis.shape == k_vis.shape and v_txt.shape == k_txt.shape
    assert k_txt.shape == (B, Hkv, Nt, D)
    assert len({a.dtype for a in (q, k_vis, v_vis, k_txt, v_txt)}) == 1
    idx = _c(idx, np.int32)
    count = _c(count, np.int32)
    k = idx.shape[2]
    assert idx.shape == (B, Hkv, k) and count.shape == (B, Hkv)
    tl = _lens(txt_len, B)
    out = np.empty((B, Hq, D), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    wsum = np.empty((B, Hq), dtype=np.float64)
    rc = _load().svo_sparse_decode_attn(B, Hq, Hkv, D, Nv, Nt, k, _dtype_code(q),
                                        default_scale(D) if scale is None else scale,
                                        _ptr(q), _ptr(k_vis), _ptr(v_vis), _ptr(k_txt), _ptr(v_txt),
                                        _ptr(tl), _ptr(idx), _ptr(count),
                                        _ptr(out), _ptr(lse), _ptr(wsum))
    if rc:
        raise ValueError(f"svo_sparse_decode_attn failed: {rc}")
    return out, lse, wsum


def decode_step(q, k_vis, v_vis, k_txt, v_txt, k: int, vis_len=None, txt_len=None,
                scale: Optional[float] = None) -> dict:
    """Steps 1-3 chained.  Returns dict(scores, idx, count, out, lse, wsum)."""
    q, k_vis, v_vis, k_txt, v_txt = map(_c, (q, k_vis, v_vis, k_txt, v_txt))
    B, Hq, D = q.shape
    _, Hkv, Nv, _ = k_vis.shape
    Nt = k_txt.shape[2]
    assert v_vis.shape == k_vis.shape and v_txt.shape == k_txt.shape
    assert len({a.dtype for a in (q, k_vis, v_vis, k_txt, v_txt)}) == 1
    vl, tl = _lens(vis_len, B), _lens(txt_len, B)
    scores = np.empty((B, Hkv, Nv), dtype=np.float64)
    idx = np.full((B, Hkv, max(k, 0)), -1, dtype=np.int32)
    cnt = np.zeros((B, Hkv), dtype=np.int32)
    out = np.empty((B, Hq, D), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    wsum = np.empty((B, Hq), dtype=np.float64)
    rc = _load().svo_decode_step(B, Hq, Hkv, D, Nv, Nt, k, _dtype_code(q),
                                 default_scale(D) if scale is None else scale,
                                 _ptr(q), _ptr(k_vis), _ptr(v_vis), _ptr(k_txt), _ptr(v_txt),
                                 _ptr(vl), _ptr(tl), _ptr(scores), _ptr(idx), _ptr(cnt),
                                 _ptr(out), _ptr(lse), _ptr(wsum))
    if rc:
        raise ValueError(f"svo_decode_step failed: {rc}")
    return dict(scores=scores, idx=idx, count=cnt, out=out, lse=lse, wsum=wsum)


def pack_selected(k_vis, v_vis, idx, count):
    """Packing of the kept rows (paper section 3.2: the selected visual KV entries are packed into a
    contiguous region), written out as its definition with plain loops:
    k_pack[b,g,i,:] = k_vis[b,g,idx[b,g,i],:] for i < count[b,g], zero rows after that."""
    k_vis, v_vis = _c(k_vis), _c(v_vis)
    idx, count = _c(idx, np.int32), _c(count, np.int32)
    B, Hkv, Nv, D = k_vis.shape
    k = idx.shape[2]
    k_pack = np.zeros((B, Hkv, k, D), dtype=k_vis.dtype)
    v_pack = np.zeros((B, Hkv, k, D), dtype=v_vis.dtype)
    for b in range(B):
        for g in range(Hkv):
            for i in range(int(count[b, g])):
                j = int(idx[b, g, i])
                assert 0 <= j < Nv
                k_pack[b, g, i, :] = k_vis[b, g, j, :]
                v_pack[b, g, i, :] = v_vis[b, g, j, :]
    return k_pack, v_pack


def score_visual_mass(q_multi, k_vis, k_txt, vis_len=None, txt_len=None, scale: Optional[float] = None):
    """Attention mass of a multi-token query on every visual key (paper section 3.2, "Query-Aware Token
    Selection": aggregate attention strength between the query embeddings and the visual entries of the
    KV cache), written out as its definition in float64 with the attention matrix formed explicitly:
    row (i, h) -- query token i (text row txt_len - Tq + i), head h -- takes one softmax over the text
    rows up to and including its own and all live visual rows; mass[b,g,j] is the sum of the rows'
    probabilities of visual key j over the query tokens and the heads of group g.
    Returns (mass [B,Hkv,Nv] float64 with -inf past vis_len, lse [B,Tq,Hq] float64)."""
    q = _c(q_multi).astype(np.float64)
    kv = _c(k_vis).astype(np.float64)
    kt = _c(k_txt).astype(np.float64)
    B, Tq, Hq, D = q.shape
    _, Hkv, Nv, _ = kv.shape
    Nt = kt.shape[2]
    G = Hq // Hkv
    sc = default_scale(D) if scale is None else scale
    vl = np.full(B, Nv) if vis_len is None else np.asarray(vis_len)
    tl = np.full(B, Nt) if txt_len is None else np.asarray(txt_len)
    mass = np.full((B, Hkv, Nv), -np.inf)
    lse = np.full((B, Tq, Hq), np.inf)
    for b in range(B):
        nv, nt = int(vl[b]), int(tl[b])
        mass[b, :, :nv] = 0.0
        for i in range(Tq):
            n_seen_txt = min(max(nt - Tq + i + 1, 0), nt)
            for h in range(Hq):
                g = h // G
                logit_t = sc * (kt[b, g, :n_seen_txt] @ q[b, i, h])
                logit_v = sc * (kv[b, g, :nv] @ q[b, i, h])
                allv = np.concatenate([logit_t, logit_v])
                if allv.size == 0:
                    continue
                m = allv.max()
                z = np.exp(allv - m).sum()
                lse[b, i, h] = m + np.log(z)
                mass[b, g, :nv] += np.exp(logit_v - m) / z
    return mass, lse


def salience_self(q_all, k_all, vis_len=None, scale: Optional[float] = None):
    """Query-agnostic salience of the tokens of a vision-encoder layer that has no summary token (paper
    section 3.1, "Token Salience Estimation": importance is the intra-visual attention averaged over
    all tokens), written out as its definition in float64 with the attention matrix formed explicitly:
    per head, every token's query row takes one softmax over all live tokens' keys; salience[b, j] is the
    probability that key j receives, averaged over the query tokens and the heads.
    q_all [B, N, H, D], k_all [B, H, N, D]; tokens at or past vis_len[b] neither ask nor are seen.
    Returns (salience [B, N] float64 with -inf past vis_len, lse [B, N, H] float64 with +inf past vis_len)."""
    q = _c(q_all).astype(np.float64)
    k = _c(k_all).astype(np.float64)
    B, N, H, D = q.shape
    assert k.shape == (B, H, N, D)
    sc = default_scale(D) if scale is None else scale
    vl = np.full(B, N) if vis_len is None else np.asarray(vis_len)
    sal = np.full((B, N), -np.inf)
    lse = np.full((B, N, H), np.inf)
    for b in range(B):
        n = int(vl[b])
        if n == 0:
            continue
        total = np.zeros(n)
        for h in range(H):
            logits = sc * (q[b, :n, h] @ k[b, h, :n].T)          # [query token, key token]
            m = logits.max(axis=1, keepdims=True)
            e = np.exp(logits - m)
            z = e.sum(axis=1, keepdims=True)
            lse[b, :n, h] = (m + np.log(z))[:, 0]
            total += (e / z).sum(axis=0)                          # attention received by each key
        sal[b, :n] = total / (H * n)
    return sal, lse
