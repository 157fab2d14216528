"""Seeded synthetic inputs for the sparse decode step (shared by tests, bench, smoke).

This module only DRAWS inputs; it holds none of the method's arithmetic (no
scoring, no selection, no softmax) and is imported by neither the HIP binding
nor the CPU oracle.  Both sides consume the same bits produced here.

Workloads follow the paper's decode setting (section 4.1: batch 1, one GPU;
table "video understanding": 256-frame inputs at decode sparsity 0.90-0.95;
section 4.5: GQA backbones such as the 28-query/4-kv-head, 28-layer one used
by LongVILA-7B and Qwen2.5-VL-7B).  The paper's datasets are not available, so
Gaussian tensors of those shapes stand in for real KV caches:

  cfg 1  tiny:   B1, 4q/1kv, D64, fp32, 512 visual + 64 text, k=64, iid N(0,1)
  cfg 2  image:  B1, 28q/4kv, D128, fp16, 3136 visual + 256 text, k=784, iid N(0,1)
  cfg 3  video:  28 layers, 12544 visual + 512 text, k=1254; 5 % of the visual
                 keys of every (layer, kv head) are shifted by +2 along the unit
                 vector of that group's summed query (planted salient tokens)
  cfg 4  long video: 28 layers, 256 frames x 196 = 50176 visual + 1024 text,
                 k=2509; every frame adds its own offset vector ~ N(0, 0.5^2 I)
                 to its K rows and another one to its V rows
  cfg 5  batched multi-turn: B16, visual length ~ U{4096..8192} per sequence,
                 capacity 8192 (padding rows hold the sentinel 1e4), 1024 text,
                 k=512; 4 rounds, each with a fresh query

Recipe: one numpy Generator per layer, seed = 20251017 + 1000*cfg + layer; draw
float32 standard normals in the order q, K_vis, V_vis, K_txt, V_txt, then the
structure variables; add structure in float32; cast once to the config dtype
(round to nearest even).  Layers are folded into the batch dimension.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

BASE_SEED = 20251017
PAD_SENTINEL = 1.0e4


@dataclass(frozen=True)
class Workload:
    cfg: int
    name: str
    batch: int          # sequences per layer
    layers: int         # independent layers, folded into the batch dimension
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str          # "f16" | "f32"
    n_vis: int          # capacity of the visual segment
    n_txt: int
    k: int
    structure: str      # "iid" | "planted" | "frames" | "ragged"
    frame_len: int = 196
    vis_len_min: int = 0  # ragged only
    rounds: int = 1
    seed_offset: int = 0  # added to every seed: other draws of the same workload (bench --seed, rotating copies)

    @property
    def B(self) -> int:
        return self.batch * self.layers

    @property
    def np_dtype(self):
        return np.float16 if self.dtype == "f16" else np.float32

    @property
    def elem_size(self) -> int:
        return 2 if self.dtype == "f16" else 4


WORKLOADS: Dict[int, Workload] = {
    1: Workload(1, "tiny_fp32", 1, 1, 4, 1, 64, "f32", 512, 64, 64, "iid"),
    2: Workload(2, "image_3136", 1, 1, 28, 4, 128, "f16", 3136, 256, 784, "iid"),
    3: Workload(3, "video_64f_x28", 1, 28, 28, 4, 128, "f16", 12544, 512, 1254, "planted"),
    4: Workload(4, "longvideo_256f_x28", 1, 28, 28, 4, 128, "f16", 50176, 1024, 2509, "frames"),
    5: Workload(5, "batched_multiturn", 16, 1, 28, 4, 128, "f16", 8192, 1024, 512, "ragged",
                vis_len_min=4096, rounds=4),
}


def workload(cfg: int, **overrides) -> Workload:
    """A config, optionally shrunk (same structure, smaller sizes) for CPU-speed tests."""
    w = WORKLOADS[cfg]
    return replace(w, **overrides) if overrides else w


def _layer_rng(w: Workload, layer: int) -> np.random.Generator:
    return np.random.default_rng(BASE_SEED + w.seed_offset + 1000 * w.cfg + layer)


def _normal(rng, shape):
    return rng.standard_normal(shape, dtype=np.float32)


def make_layer(w: Workload, layer: int) -> Dict[str, np.ndarray]:
    """Inputs of one layer: q [b,Hq,D], K/V_vis [b,Hkv,Nv,D], K/V_txt [b,Hkv,Nt,D], lens."""
    rng = _layer_rng(w, layer)
    b, Hq, Hkv, D, Nv, Nt = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_vis, w.n_txt
    G = Hq // Hkv
    q = _normal(rng, (b, Hq, D))
    k_vis = _normal(rng, (b, Hkv, Nv, D))
    v_vis = _normal(rng, (b, Hkv, Nv, D))
    k_txt = _normal(rng, (b, Hkv, Nt, D))
    v_txt = _normal(rng, (b, Hkv, Nt, D))
    vis_len = np.full((b,), Nv, dtype=np.int32)
    txt_len = np.full((b,), Nt, dtype=np.int32)

    if w.structure == "planted":
        # 5 % of the keys of each (sequence, kv head) move +2 (two standard
        # deviations of a key component) along the direction of the group's
        # summed query, taken after the query is rounded to the config dtype.
        n_plant = int(0.05 * Nv)
        qd = q.astype(w.np_dtype).astype(np.float32)
        for bi in range(b):
            for g in range(Hkv):
                u = qd[bi, g * G:(g + 1) * G].sum(axis=0)
                u = u / np.linalg.norm(u)
                pos = rng.choice(Nv, size=n_plant, replace=False)
                k_vis[bi, g, pos, :] += np.float32(2.0) * u.astype(np.float32)
    elif w.structure == "frames":
        F = -(-Nv // w.frame_len)
        for bi in range(b):
            for g in range(Hkv):
                mu_k = np.float32(0.5) * _normal(rng, (F, D))
                mu_v = np.float32(0.5) * _normal(rng, (F, D))
                k_vis[bi, g] += np.repeat(mu_k, w.frame_len, axis=0)[:Nv]
                v_vis[bi, g] += np.repeat(mu_v, w.frame_len, axis=0)[:Nv]
    elif w.structure == "ragged":
        vis_len = rng.integers(w.vis_len_min, Nv, size=(b,), endpoint=True).astype(np.int32)
        for bi in range(b):
            k_vis[bi, :, vis_len[bi]:, :] = PAD_SENTINEL
            v_vis[bi, :, vis_len[bi]:, :] = PAD_SENTINEL
    elif w.structure != "iid":
        raise ValueError(w.structure)

    dt = w.np_dtype
    return dict(q=q.astype(dt), k_vis=k_vis.astype(dt), v_vis=v_vis.astype(dt),
                k_txt=k_txt.astype(dt), v_txt=v_txt.astype(dt),
                vis_len=vis_len, txt_len=txt_len)


def make_inputs(w: Workload, layers: Optional[range] = None, workers: int = 1) -> Dict[str, np.ndarray]:
    """All (or a range of) layers folded into the batch dimension, layer-major.

    Layers have independent seeds, so drawing them on several threads gives the same bits."""
    layers = range(w.layers) if layers is None else layers
    if workers > 1 and len(layers) > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=workers) as ex:
            parts = list(ex.map(lambda l: make_layer(w, l), layers))
    else:
        parts = [make_layer(w, l) for l in layers]
    if len(parts) == 1:
        return parts[0]
    return {key: np.concatenate([p[key] for p in parts], axis=0) for key in parts[0]}


def round_query(w: Workload, rnd: int) -> np.ndarray:
    """Fresh query of conversation round rnd >= 1 (round 0 uses make_inputs' q)."""
    rng = np.random.default_rng(BASE_SEED + w.seed_offset + 1000 * w.cfg + 500 + rnd)
    return _normal(rng, (w.B, w.n_q_heads, w.head_dim)).astype(w.np_dtype)


def cache_bytes(w: Workload) -> int:
    """Bytes of the whole KV cache of the workload (visual and text, K and V, at capacity)."""
    return int(2 * w.B * w.n_kv_heads * (w.n_vis + w.n_txt) * w.head_dim * w.elem_size)


def algorithmic_bytes(w: Workload, vis_len: np.ndarray, txt_len: np.ndarray) -> int:
    """Bytes the method itself must move in one step: every visual K row once, plus
    K and V rows of the selected visual tokens and of every text token."""
    kb = np.minimum(w.k, vis_len.astype(np.int64))
    per_b = vis_len.astype(np.int64) + 2 * kb + 2 * txt_len.astype(np.int64)
    return int(w.n_kv_heads * w.head_dim * w.elem_size * per_b.sum())
