"""Property tests of the CPU oracle over drawn shapes and values (hypothesis): the pins of
test_oracle_pins.py hold on fixed cases; here the same kind of statement -- brute force, a library
routine, an invariant -- is checked on shapes nobody chose by hand, ties and ragged lengths included."""
import numpy as np
import torch
from hypothesis import given, settings, strategies as st

import oracle

SET = settings(max_examples=40, deadline=None)


@SET
@given(st.integers(1, 60), st.integers(0, 70), st.integers(1, 5), st.integers(0, 2 ** 31 - 1))
def test_topk_is_the_brute_force_sort_with_ties_toward_the_lower_index(n, k, levels, seed):
    rng = np.random.default_rng(seed)
    B, H = 2, 2
    s = rng.integers(0, levels, size=(B, H, n)).astype(np.float64)     # few distinct values: heavy ties
    s[rng.random(s.shape) < 0.1] = -np.inf                            # masked scores lose against everything finite
    vis_len = rng.integers(0, n, size=B, endpoint=True).astype(np.int32)
    idx, cnt = oracle.topk_select(s, k, vis_len)
    for b in range(B):
        nb = int(vis_len[b])
        kb = min(k, nb)
        for h in range(H):
            order = np.lexsort((np.arange(nb), -s[b, h, :nb]))          # score descending, index ascending
            want = np.sort(order[:kb])
            assert cnt[b, h] == kb
            assert idx[b, h, :kb].tolist() == want.tolist()
            assert np.all(idx[b, h, kb:] == -1)


@SET
@given(st.integers(1, 3), st.integers(1, 3), st.integers(1, 4), st.sampled_from([8, 16]), st.integers(1, 25),
       st.integers(0, 9), st.sampled_from([np.float16, np.float32]), st.integers(0, 2 ** 31 - 1))
def test_keeping_everything_is_dense_attention_by_the_library(B, Hkv, G, D, Nv, Nt, dtype, seed):
    rng = np.random.default_rng(seed)
    f = lambda *s: rng.standard_normal(s).astype(dtype)
    q, kv, vv, kt, vt = f(B, Hkv * G, D), f(B, Hkv, Nv, D), f(B, Hkv, Nv, D), f(B, Hkv, Nt, D), f(B, Hkv, Nt, D)
    r = oracle.decode_step(q, kv, vv, kt, vt, Nv + 3)
    assert np.all(r["count"] == Nv)
    K = torch.from_numpy(np.concatenate([kt, kv], axis=2).astype(np.float64)).repeat_interleave(G, dim=1)
    V = torch.from_numpy(np.concatenate([vt, vv], axis=2).astype(np.float64)).repeat_interleave(G, dim=1)
    Q = torch.from_numpy(q.astype(np.float64))[:, :, None, :]
    want = torch.nn.functional.scaled_dot_product_attention(Q, K, V)[:, :, 0, :].numpy()
    assert np.abs(r["out"] - want).max() <= 1e-12
    assert np.abs(r["wsum"] - 1.0).max() <= 1e-12


@SET
@given(st.integers(1, 3), st.integers(1, 2), st.integers(1, 3), st.integers(2, 30), st.integers(0, 8), st.integers(0, 12),
       st.integers(0, 2 ** 31 - 1))
def test_attention_over_a_kept_set_splits_and_merges_by_log_sum_exp(B, Hkv, G, Nv, Nt, k, seed):
    """The step's output over text + kept tokens equals the log-sum-exp merge of attention over the text alone and
    over the kept visual tokens alone (what the GPU's chunked path relies on), for any kept set the step picks."""
    rng = np.random.default_rng(seed)
    D = 8
    f = lambda *s: rng.standard_normal(s).astype(np.float32)
    q, kv, vv, kt, vt = f(B, Hkv * G, D), f(B, Hkv, Nv, D), f(B, Hkv, Nv, D), f(B, Hkv, Nt, D), f(B, Hkv, Nt, D)
    r = oracle.decode_step(q, kv, vv, kt, vt, k)
    o_t, l_t, _ = oracle.sparse_decode_attn(q, kv, vv, kt, vt, r["idx"], np.zeros_like(r["count"]))        # text alone
    empty = kt[:, :, :0]
    o_v, l_v, _ = oracle.sparse_decode_attn(q, kv, vv, empty, empty, r["idx"], r["count"])                   # kept alone
    with np.errstate(invalid="ignore", divide="ignore"):
        m = np.maximum(l_t, l_v)
        wt, wv = np.exp(l_t - m), np.exp(l_v - m)
        wt, wv = np.where(np.isfinite(l_t), wt, 0.0), np.where(np.isfinite(l_v), wv, 0.0)
        merged = (wt[..., None] * np.nan_to_num(o_t) + wv[..., None] * np.nan_to_num(o_v)) / (wt + wv)[..., None]
        lse = m + np.log(wt + wv)
    live = np.isfinite(r["lse"])
    assert np.array_equal(live, np.isfinite(lse))
    assert np.abs(merged - r["out"])[live].max(initial=0.0) <= 1e-12
    assert np.abs(lse - r["lse"])[live].max(initial=0.0) <= 1e-12
