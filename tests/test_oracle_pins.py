"""Pins of the CPU oracle against things other than itself (CPU only).

Each test fixes one part of the oracle to what the mathematics or a library
routine says, chosen so that a dropped term, a wrong sign or index, or a
transposed operand fails at least one of them:

  whole step : k = Nv reproduces dense attention (library SDPA in float64);
               hand-worked example (tests/golden/worked_step_2heads.txt)
  attention  : identical keys -> mean of V; softmax mass = 1; dominant key ->
               its V row; key-shift invariance; V-scaling; LSE split/merge
  selection  : brute-force lexsort; set properties; all-equal; monotone in k;
               hand-worked tie cases (tests/golden/topk_ties.txt)
  scoring    : linearity closed form; G = 1 is the plain logit; unit-vector
               query reads the key matrix back
  order      : permutation of the visual / text cache rows
  ragged     : padding rows are never read; k = 0, Nt = 0, k >= Nv
  widening   : all 65536 binary16 patterns against numpy's float16 -> float64
  mass       : library softmax of the masked matrix; probability conservation; Tq = G = 1 is the attention weight;
               hand-worked causal offsets (tests/golden/mass_causal_2q_3t.txt)
  salience   : library attention with V = I; two-token logistic closed form; one shared query -> its softmax;
               uniform / conservation / key-shift / permutation invariants; dominant key
"""
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_case(seed, B=2, Hq=4, Hkv=2, D=16, Nv=40, Nt=9, dtype=np.float32):
    rng = np.random.default_rng(seed)
    f = lambda *s: rng.standard_normal(s).astype(dtype)
    return dict(q=f(B, Hq, D), k_vis=f(B, Hkv, Nv, D), v_vis=f(B, Hkv, Nv, D),
                k_txt=f(B, Hkv, Nt, D), v_txt=f(B, Hkv, Nt, D))


def dense_reference(c, scale=None):
    """Library routine: float64 SDPA over text followed by ALL visual tokens."""
    q = torch.from_numpy(c["q"].astype(np.float64))
    B, Hq, D = q.shape
    Hkv = c["k_vis"].shape[1]
    G = Hq // Hkv
    K = torch.from_numpy(np.concatenate([c["k_txt"], c["k_vis"]], axis=2).astype(np.float64))
    V = torch.from_numpy(np.concatenate([c["v_txt"], c["v_vis"]], axis=2).astype(np.float64))
    K = K.repeat_interleave(G, dim=1)
    V = V.repeat_interleave(G, dim=1)
    o = torch.nn.functional.scaled_dot_product_attention(q[:, :, None, :], K, V, scale=scale)
    return o[:, :, 0, :].numpy()


# ---------------------------------------------------------------- widening
def test_half_widening_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


# ---------------------------------------------------------------- whole step
@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("shape", [dict(B=2, Hq=4, Hkv=2, D=16, Nv=40, Nt=9),
                                   dict(B=1, Hq=7, Hkv=1, D=32, Nv=33, Nt=0),
                                   dict(B=3, Hq=6, Hkv=6, D=8, Nv=17, Nt=5)])
def test_k_equals_nv_is_dense_attention(dtype, shape):
    c = rand_case(1, dtype=dtype, **shape)
    r = oracle.decode_step(k=shape["Nv"], **c)
    assert np.array_equal(r["count"], np.full_like(r["count"], shape["Nv"]))
    assert np.array_equal(r["idx"][0, 0], np.arange(shape["Nv"]))
    np.testing.assert_allclose(r["out"], dense_reference(c), rtol=0, atol=1e-12)


def test_explicit_scale_is_used_by_all_steps():
    c = rand_case(2)
    r = oracle.decode_step(k=40, scale=0.37, **c)
    np.testing.assert_allclose(r["out"], dense_reference(c, scale=0.37), atol=1e-12)
    s1 = oracle.score_visual(c["q"], c["k_vis"], scale=1.0)
    np.testing.assert_allclose(r["scores"], 0.37 * s1, rtol=1e-14)


def test_worked_example_from_golden_file():
    vals = {}
    for line in open(os.path.join(GOLDEN, "worked_step_2heads.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *nums = line.split()
        vals[key] = np.array([float(x) for x in nums])
    q = np.array([[[1, 0], [0, 1]]], dtype=np.float32)
    k_vis = np.array([[[[1, 0], [0, 3], [2, 2], [-1, -1]]]], dtype=np.float32)
    v_vis = np.array([[[[9, 9], [0, 4], [2, -2], [7, 7]]]], dtype=np.float32)
    k_txt = np.array([[[[0, 0]]]], dtype=np.float32)
    v_txt = np.array([[[[1, 1]]]], dtype=np.float32)
    r = oracle.decode_step(q, k_vis, v_vis, k_txt, v_txt, k=2, scale=1.0)
    np.testing.assert_allclose(r["scores"][0, 0], vals["scores"], atol=1e-15)
    assert r["idx"][0, 0].tolist() == vals["idx"].astype(int).tolist()
    np.testing.assert_allclose(r["out"][0, 0], vals["out0"], rtol=1e-14)
    np.testing.assert_allclose(r["out"][0, 1], vals["out1"], rtol=1e-14)
    np.testing.assert_allclose(r["lse"][0], vals["lse"], rtol=1e-14)


# ---------------------------------------------------------------- attention
def test_identical_keys_give_mean_of_values():
    c = rand_case(3, Nv=30, Nt=6)
    key = c["k_vis"][:, :, :1, :].copy()
    c["k_vis"][:] = key
    c["k_txt"][:] = key
    r = oracle.decode_step(k=10, **c)
    G = c["q"].shape[1] // c["k_vis"].shape[1]
    for b in range(2):
        for h in range(4):
            g = h // G
            rows = np.concatenate([c["v_txt"][b, g], c["v_vis"][b, g, r["idx"][b, g]]], axis=0)
            np.testing.assert_allclose(r["out"][b, h], rows.astype(np.float64).mean(axis=0),
                                       atol=1e-13)
    # all scores tie, so the kept set is the first k indices
    assert np.array_equal(r["idx"][0, 0], np.arange(10))


def test_softmax_mass_is_one():
    for seed, dtype in [(4, np.float32), (5, np.float16)]:
        c = rand_case(seed, Nv=300, Nt=50, D=64, dtype=dtype)
        c["q"] = (c["q"] * 6).astype(dtype)   # peaky logits as well
        r = oracle.decode_step(k=75, **c)
        assert np.all(np.abs(r["wsum"] - 1.0) < 1e-6)
        assert np.all(np.abs(r["wsum"] - 1.0) < 1e-12)


def test_dominant_key_returns_its_value_row():
    c = rand_case(6, B=1, Hq=2, Hkv=1, D=16, Nv=20, Nt=4)
    u = c["q"][0].astype(np.float64).sum(axis=0)
    # key 7 is strongly aligned with both heads' queries
    c["q"][0, 1] = c["q"][0, 0]
    c["k_vis"][0, 0, 7] = (40.0 * c["q"][0, 0] / np.linalg.norm(c["q"][0, 0])).astype(np.float32)
    r = oracle.decode_step(k=3, **c)
    assert 7 in r["idx"][0, 0]
    scale = 1 / 4.0
    logits_other = scale * np.abs(c["q"][0, 0].astype(np.float64)
                                  @ np.concatenate([c["k_vis"][0, 0], c["k_txt"][0, 0]]).T.astype(np.float64))
    top = scale * 40.0 * np.linalg.norm(c["q"][0, 0].astype(np.float64))
    others = np.sort(logits_other)[:-1].max()
    bound = 7 * np.exp(others - top) * 2 * np.abs(np.concatenate([c["v_vis"], c["v_txt"]], axis=2)).max()
    assert bound < 1e-3
    assert np.abs(r["out"][0, 0] - c["v_vis"][0, 0, 7]).max() <= bound
    del u


def test_adding_a_vector_to_every_key_changes_nothing():
    c = rand_case(7, dtype=np.float32)
    # exactly representable shift so that the shifted keys are exact in fp32
    for a in ("k_vis", "k_txt", "q"):
        c[a] = np.round(c[a] * 64) / 64
    shift = (np.round(np.random.default_rng(70).standard_normal(16) * 8) / 8).astype(np.float32)
    r0 = oracle.decode_step(k=11, **c)
    c2 = dict(c, k_vis=c["k_vis"] + shift, k_txt=c["k_txt"] + shift)
    r1 = oracle.decode_step(k=11, **c2)
    assert np.array_equal(r0["idx"], r1["idx"])
    np.testing.assert_allclose(r0["out"], r1["out"], atol=1e-12)
    # every score of a group moves by the same amount: scale * <sum_h q_h, shift>
    G = 2
    for g in range(2):
        d = (r1["scores"] - r0["scores"])[0, g]
        want = 0.25 * (c["q"][0, g * G:(g + 1) * G].astype(np.float64).sum(0) @ shift.astype(np.float64))
        np.testing.assert_allclose(d, want, atol=1e-12)


def test_scaling_values_scales_output():
    c = rand_case(8)
    r0 = oracle.decode_step(k=13, **c)
    c2 = dict(c, v_vis=c["v_vis"] * np.float32(-4), v_txt=c["v_txt"] * np.float32(-4))
    r1 = oracle.decode_step(k=13, **c2)
    np.testing.assert_allclose(r1["out"], -4 * r0["out"], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(r1["lse"], r0["lse"], rtol=0, atol=0)


def test_lse_merge_of_text_part_and_visual_part_reproduces_the_whole():
    c = rand_case(9, Nv=50, Nt=12)
    whole = oracle.decode_step(k=20, **c)
    idx, cnt = whole["idx"], whole["count"]
    B, Hkv = cnt.shape
    txt_only = oracle.sparse_decode_attn(c["q"], c["k_vis"], c["v_vis"], c["k_txt"], c["v_txt"],
                                         idx, np.zeros_like(cnt))
    vis_only = oracle.sparse_decode_attn(c["q"], c["k_vis"], c["v_vis"], c["k_txt"], c["v_txt"],
                                         idx, cnt, txt_len=np.zeros(B, np.int32))
    (o1, l1, _), (o2, l2, _) = txt_only, vis_only
    m = np.maximum(l1, l2)
    a1, a2 = np.exp(l1 - m), np.exp(l2 - m)
    merged = (a1[..., None] * o1 + a2[..., None] * o2) / (a1 + a2)[..., None]
    np.testing.assert_allclose(merged, whole["out"], atol=1e-13)
    np.testing.assert_allclose(m + np.log(a1 + a2), whole["lse"], atol=1e-13)


def test_lse_is_log_sum_exp_of_logits():
    c = rand_case(10, B=1, Hq=1, Hkv=1, D=8, Nv=6, Nt=3)
    r = oracle.decode_step(k=6, **c)
    keys = np.concatenate([c["k_txt"][0, 0], c["k_vis"][0, 0]]).astype(np.float64)
    logits = keys @ c["q"][0, 0].astype(np.float64) / np.sqrt(8.0)
    import scipy.special
    np.testing.assert_allclose(r["lse"][0, 0], scipy.special.logsumexp(logits), rtol=1e-14)


# ---------------------------------------------------------------- selection
@pytest.mark.parametrize("seed", range(6))
def test_selection_matches_brute_force_lexsort(seed):
    rng = np.random.default_rng(100 + seed)
    B, Hkv, Nv = 2, 3, int(rng.integers(1, 60))
    k = int(rng.integers(0, Nv + 3))
    # few distinct values -> many ties
    s = rng.integers(-3, 4, size=(B, Hkv, Nv)).astype(np.float64) / 2
    vis_len = rng.integers(0, Nv, size=B, endpoint=True).astype(np.int32)
    idx, cnt = oracle.topk_select(s, k, vis_len)
    for b in range(B):
        n = int(vis_len[b])
        kb = min(k, n)
        for g in range(Hkv):
            order = np.lexsort((np.arange(n), -s[b, g, :n]))   # primary: -s, secondary: index
            want = np.sort(order[:kb])
            assert cnt[b, g] == kb
            assert np.array_equal(idx[b, g, :kb], want)
            assert np.all(idx[b, g, kb:] == -1)


def test_selection_set_properties_and_monotone_in_k():
    rng = np.random.default_rng(11)
    s = rng.standard_normal((1, 1, 500))
    prev = set()
    for k in (0, 1, 7, 8, 100, 499, 500):
        idx, cnt = oracle.topk_select(s, k)
        sel = idx[0, 0, :cnt[0, 0]]
        assert cnt[0, 0] == k and len(set(sel.tolist())) == k
        assert np.all(np.diff(sel) > 0) and (k == 0 or (sel[0] >= 0 and sel[-1] < 500))
        inside = s[0, 0, sel]
        outside = np.delete(s[0, 0], sel)
        if 0 < k < 500:
            assert inside.min() > outside.max()
        assert prev <= set(sel.tolist())
        prev = set(sel.tolist())


def test_all_equal_scores_keep_the_first_k():
    s = np.full((2, 2, 64), 1.25)
    idx, cnt = oracle.topk_select(s, 10)
    assert np.array_equal(idx, np.broadcast_to(np.arange(10, dtype=np.int32), (2, 2, 10)))
    assert np.all(cnt == 10)


def test_topk_golden_tie_cases():
    for line in open(os.path.join(GOLDEN, "topk_ties.txt")):
        if line.startswith("#") or not line.strip():
            continue
        s_txt, k_txt, want_txt = line.split("|")
        s = np.array([float(x) for x in s_txt.split()])[None, None, :]
        k = int(k_txt)
        want = [int(x) for x in want_txt.split()]
        idx, cnt = oracle.topk_select(s, k)
        assert cnt[0, 0] == len(want), line
        assert idx[0, 0, :cnt[0, 0]].tolist() == want, line
        assert np.all(idx[0, 0, cnt[0, 0]:] == -1)


# ---------------------------------------------------------------- scoring
@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_score_equals_scaled_dot_with_summed_query(dtype):
    c = rand_case(12, B=2, Hq=14, Hkv=2, D=32, Nv=25, dtype=dtype)
    s = oracle.score_visual(c["q"], c["k_vis"])
    qs = c["q"].astype(np.float64).reshape(2, 2, 7, 32).sum(axis=2)
    want = np.einsum("bgd,bgnd->bgn", qs, c["k_vis"].astype(np.float64)) / np.sqrt(32.0)
    np.testing.assert_allclose(s, want, rtol=0, atol=1e-13)


def test_score_with_one_head_per_group_is_the_attention_logit():
    c = rand_case(13, B=1, Hq=3, Hkv=3, D=8, Nv=10)
    s = oracle.score_visual(c["q"], c["k_vis"])
    want = np.einsum("hd,hnd->hn", c["q"][0].astype(np.float64), c["k_vis"][0].astype(np.float64)) / np.sqrt(8.0)
    np.testing.assert_allclose(s[0], want, atol=1e-14)


def test_unit_vector_query_reads_back_the_key_matrix():
    B, Hq, Hkv, D, Nv = 2, 6, 3, 8, 12
    k_vis = np.arange(B * Hkv * Nv * D, dtype=np.float32).reshape(B, Hkv, Nv, D)
    for b, g, hh, d in [(0, 0, 0, 0), (1, 2, 1, 5), (0, 1, 1, 7), (1, 0, 0, 3)]:
        q = np.zeros((B, Hq, D), dtype=np.float32)
        q[b, g * 2 + hh, d] = 1.0
        s = oracle.score_visual(q, k_vis, scale=1.0)
        want = np.zeros((B, Hkv, Nv))
        want[b, g] = k_vis[b, g, :, d]
        assert np.array_equal(s, want)


# ---------------------------------------------------------------- order invariance
def test_permuting_the_visual_cache_maps_the_set_and_keeps_the_output():
    c = rand_case(14, Nv=64, Nt=10)
    r0 = oracle.decode_step(k=16, **c)
    perm = np.random.default_rng(140).permutation(64)
    c2 = dict(c, k_vis=c["k_vis"][:, :, perm], v_vis=c["v_vis"][:, :, perm])
    r1 = oracle.decode_step(k=16, **c2)
    np.testing.assert_allclose(r1["out"], r0["out"], atol=1e-12)
    np.testing.assert_allclose(r1["lse"], r0["lse"], atol=1e-12)
    for b in range(2):
        for g in range(2):
            assert set(perm[r1["idx"][b, g]].tolist()) == set(r0["idx"][b, g].tolist())


def test_permuting_the_text_cache_keeps_the_output():
    c = rand_case(15, Nv=30, Nt=20)
    r0 = oracle.decode_step(k=8, **c)
    perm = np.random.default_rng(150).permutation(20)
    c2 = dict(c, k_txt=c["k_txt"][:, :, perm], v_txt=c["v_txt"][:, :, perm])
    r1 = oracle.decode_step(k=8, **c2)
    assert np.array_equal(r1["idx"], r0["idx"])
    np.testing.assert_allclose(r1["out"], r0["out"], atol=1e-12)


# ---------------------------------------------------------------- ragged / edges
def test_padding_rows_are_never_read():
    c = rand_case(16, B=3, Nv=40, Nt=12)
    vis_len = np.array([40, 17, 0], np.int32)
    txt_len = np.array([12, 5, 3], np.int32)
    r0 = oracle.decode_step(k=20, vis_len=vis_len, txt_len=txt_len, **c)
    c2 = {a: v.copy() for a, v in c.items()}
    for b in range(3):
        c2["k_vis"][b, :, vis_len[b]:] = 1e30
        c2["v_vis"][b, :, vis_len[b]:] = np.nan
        c2["k_txt"][b, :, txt_len[b]:] = 1e30
        c2["v_txt"][b, :, txt_len[b]:] = np.nan
    r1 = oracle.decode_step(k=20, vis_len=vis_len, txt_len=txt_len, **c2)
    assert np.array_equal(r0["idx"], r1["idx"])
    assert np.array_equal(r0["count"], np.array([[20, 20], [17, 17], [0, 0]]))
    np.testing.assert_array_equal(r0["out"], r1["out"])
    assert np.all(np.isneginf(r0["scores"][1, :, 17:])) and np.all(np.isfinite(r0["scores"][1, :, :17]))
    # the ragged result equals the result on the truncated, un-padded sequence
    for b in range(3):
        cb = dict(q=c["q"][b:b + 1], k_vis=c["k_vis"][b:b + 1, :, :vis_len[b]],
                  v_vis=c["v_vis"][b:b + 1, :, :vis_len[b]],
                  k_txt=c["k_txt"][b:b + 1, :, :txt_len[b]], v_txt=c["v_txt"][b:b + 1, :, :txt_len[b]])
        rb = oracle.decode_step(k=20, **cb)
        np.testing.assert_allclose(rb["out"][0], r0["out"][b], atol=1e-14)


def test_k_zero_is_text_only_and_nt_zero_is_visual_only():
    c = rand_case(17)
    r = oracle.decode_step(k=0, **c)
    assert r["idx"].shape == (2, 2, 0) and np.all(r["count"] == 0)
    c_txt = dict(c, k_vis=c["k_vis"][:, :, :0], v_vis=c["v_vis"][:, :, :0])
    np.testing.assert_allclose(r["out"], dense_reference(c_txt), atol=1e-13)
    c0 = dict(c, k_txt=c["k_txt"][:, :, :0], v_txt=c["v_txt"][:, :, :0])
    r = oracle.decode_step(k=1000, **c0)      # k >= Nv clamps to Nv
    assert np.all(r["count"] == 40)
    np.testing.assert_allclose(r["out"], dense_reference(c0), atol=1e-13)


def test_sparse_step_differs_from_dense_and_keeps_exactly_the_selected_rows():
    """Guards against an attention step that ignores idx: recompute with numpy on idx."""
    c = rand_case(18, B=1, Hq=4, Hkv=2, D=16, Nv=60, Nt=7)
    r = oracle.decode_step(k=9, **c)
    assert np.abs(r["out"] - dense_reference(c)).max() > 1e-3
    for h in range(4):
        g = h // 2
        keys = np.concatenate([c["k_txt"][0, g], c["k_vis"][0, g, r["idx"][0, g]]]).astype(np.float64)
        vals = np.concatenate([c["v_txt"][0, g], c["v_vis"][0, g, r["idx"][0, g]]]).astype(np.float64)
        import scipy.special
        w = scipy.special.softmax(keys @ c["q"][0, h].astype(np.float64) / 4.0)
        np.testing.assert_allclose(r["out"][0, h], w @ vals, atol=1e-13)


# ------------------------------------------------------------------ packing (section 3.2: contiguous packed region)
def test_packing_is_numpy_take_and_attention_over_the_packed_rows_is_unchanged():
    """Pins of oracle.pack_selected: (1) it equals numpy's take_along_axis (a library gather) with
    zero rows past count; (2) attention over the packed segment with the identity index list equals
    attention over the full cache with idx -- the statement that packing changes the layout only."""
    rng = np.random.default_rng(314)
    B, Hq, Hkv, D, Nv, Nt, k = 2, 6, 2, 64, 97, 13, 20
    f = lambda *s: rng.standard_normal(s).astype(np.float32)
    q, kv, vv, kt, vt = f(B, Hq, D), f(B, Hkv, Nv, D), f(B, Hkv, Nv, D), f(B, Hkv, Nt, D), f(B, Hkv, Nt, D)
    vis_len = np.array([Nv, 11], np.int32)
    st = oracle.decode_step(q, kv, vv, kt, vt, k, vis_len=vis_len)
    idx, cnt = st["idx"], st["count"]
    assert list(cnt[:, 0]) == [20, 11]
    kp, vp = oracle.pack_selected(kv, vv, idx, cnt)
    safe = np.where(idx < 0, 0, idx)
    live = (np.arange(k)[None, None, :] < cnt[:, :, None])[..., None]
    assert np.array_equal(kp, np.where(live, np.take_along_axis(kv, safe[..., None], axis=2), 0))
    assert np.array_equal(vp, np.where(live, np.take_along_axis(vv, safe[..., None], axis=2), 0))
    ident = np.broadcast_to(np.arange(k, dtype=np.int32), (B, Hkv, k)).copy()
    out_p, lse_p, _ = oracle.sparse_decode_attn(q, kp, vp, kt, vt, ident, cnt)
    assert np.abs(out_p - st["out"]).max() < 1e-13 and np.abs(lse_p - st["lse"]).max() < 1e-13


# ------------------------------------------------------------------ attention-mass retrieval (multi-token query)
def _mass_case(seed, B=2, Tq=5, Hq=6, Hkv=2, D=16, Nv=37, Nt=11):
    rng = np.random.default_rng(seed)
    f = lambda *s: rng.standard_normal(s).astype(np.float32)
    return f(B, Tq, Hq, D), f(B, Hkv, Nv, D), f(B, Hkv, Nt, D)


def test_mass_equals_column_sums_of_the_library_softmax_of_the_masked_attention_matrix():
    """The attention matrix written out, masked causally over the question's own tokens, pushed through
    scipy's softmax / logsumexp (library routines), summed over rows: the oracle must agree."""
    from scipy.special import logsumexp, softmax
    qm, kv, kt = _mass_case(1)
    B, Tq, Hq, D = qm.shape
    Hkv, Nv, Nt = kv.shape[1], kv.shape[2], kt.shape[2]
    G = Hq // Hkv
    mass, lse = oracle.score_visual_mass(qm, kv, kt)
    sc = 1.0 / np.sqrt(D)
    for b in range(B):
        for g in range(Hkv):
            keys = np.concatenate([kt[b, g], kv[b, g]]).astype(np.float64)              # [Nt + Nv, D]
            rows = qm[b, :, g * G:(g + 1) * G].astype(np.float64).reshape(Tq * G, D)    # row = i * G + hh
            logits = sc * rows @ keys.T
            tok = np.repeat(np.arange(Tq), G)[:, None]
            col = np.arange(Nt + Nv)[None, :]
            logits = np.where((col < Nt) & (col > Nt - Tq + tok), -np.inf, logits)      # text after the row's own
            p = softmax(logits, axis=1)
            assert np.allclose(mass[b, g], p[:, Nt:].sum(axis=0), rtol=1e-12, atol=1e-15)
            assert np.allclose(lse[b, :, g * G:(g + 1) * G].reshape(-1), logsumexp(logits, axis=1), rtol=1e-12)


def test_mass_conserves_probability_and_respects_lengths():
    """Every row spends probability 1: visual mass + text mass = Tq * G per kv head (text mass recomputed
    here from lse); rows past vis_len get -inf and change nothing."""
    qm, kv, kt = _mass_case(2)
    B, Tq, Hq, D = qm.shape
    Hkv, Nv, Nt = kv.shape[1], kv.shape[2], kt.shape[2]
    G = Hq // Hkv
    vis_len, txt_len = np.array([Nv, 20], np.int32), np.array([Nt, 7], np.int32)
    mass, lse = oracle.score_visual_mass(qm, kv, kt, vis_len=vis_len, txt_len=txt_len)
    assert np.all(np.isneginf(mass[1, :, 20:])) and np.all(np.isfinite(mass[1, :, :20]))
    sc = 1.0 / np.sqrt(D)
    for b in range(B):
        nt = int(txt_len[b])
        for g in range(Hkv):
            text_mass = 0.0
            for i in range(Tq):
                for h in range(g * G, (g + 1) * G):
                    seen = max(nt - Tq + i + 1, 0)
                    lt = sc * kt[b, g, :seen].astype(np.float64) @ qm[b, i, h].astype(np.float64)
                    text_mass += np.exp(lt - lse[b, i, h]).sum()
            vis_mass = mass[b, g, :vis_len[b]].sum()
            assert abs(vis_mass + text_mass - Tq * G) < 1e-10
    kv2 = kv.copy()
    kv2[1, :, 20:] = 1e4                                   # padding rows are never read
    mass2, _ = oracle.score_visual_mass(qm, kv2, kt, vis_len=vis_len, txt_len=txt_len)
    assert np.array_equal(mass2, mass)


def test_mass_of_one_token_one_head_ranks_like_the_logit_and_matches_attention_weights():
    """Tq = 1, G = 1: the mass is the decode step's own softmax weight, so (a) it orders the visual keys
    exactly like the scaled-logit score of step 1, and (b) sum_j mass_j * V_j + text part reproduces the
    oracle's dense attention output (ties the new function to the already pinned attention)."""
    rng = np.random.default_rng(3)
    B, H, D, Nv, Nt = 1, 2, 16, 30, 6
    f = lambda *s: rng.standard_normal(s).astype(np.float32)
    q, kv, vv, kt, vt = f(B, H, D), f(B, H, Nv, D), f(B, H, Nv, D), f(B, H, Nt, D), f(B, H, Nt, D)
    mass, lse = oracle.score_visual_mass(q[:, None], kv, kt)
    logit = oracle.score_visual(q, kv)
    for h in range(H):
        assert np.array_equal(np.argsort(-mass[0, h], kind="stable"), np.argsort(-logit[0, h], kind="stable"))
    dense = oracle.decode_step(q, kv, vv, kt, vt, Nv)
    assert np.allclose(lse[:, 0], dense["lse"], rtol=1e-12)
    sc = 1.0 / np.sqrt(D)
    for h in range(H):
        wt = np.exp(sc * kt[0, h].astype(np.float64) @ q[0, h].astype(np.float64) - lse[0, 0, h])
        out = wt @ vt[0, h].astype(np.float64) + mass[0, h] @ vv[0, h].astype(np.float64)
        assert np.allclose(out, dense["out"][0, h], rtol=1e-10, atol=1e-12)


def test_mass_hand_worked_causal_offsets_from_golden_file():
    """The causal offset of the question's tokens against numbers worked out by hand (ratios of small
    integers, tests/golden/mass_causal_2q_3t.txt): a question that fits the text, and one longer than
    the live text, whose first token sees no text row and where a row past txt_len lies in memory."""
    from fractions import Fraction
    ln = np.array([np.log(2.0), np.log(3.0)])
    kt = np.array([[[[1, 0], [0, 1], [2, 1]]]], dtype=np.float64)
    kv = np.array([[[[1, 1], [0, 2]]]], dtype=np.float64)
    seen = set()
    for line in open(os.path.join(GOLDEN, "mass_causal_2q_3t.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, tq, nt, q_txt, mass_txt, z_txt = [x.strip() for x in line.split("|")]
        tq, nt = int(tq), int(nt)
        q = np.array([[float(x) for x in pair.split(",")] for pair in q_txt.split()]) * ln   # [Tq, 2]
        want_mass = np.array([float(Fraction(x)) for x in mass_txt.split()])
        want_z = np.array([float(x) for x in z_txt.split()])
        assert q.shape == (tq, 2) and want_z.shape == (tq,)
        mass, lse = oracle.score_visual_mass(q[None, :, None, :], kv, kt, txt_len=np.array([nt]), scale=1.0)
        np.testing.assert_allclose(mass[0, 0], want_mass, rtol=1e-14, err_msg=name)
        np.testing.assert_allclose(np.exp(lse[0, :, 0]), want_z, rtol=1e-14, err_msg=name)
        seen.add(name)
    assert seen == {"A", "B"}


# ------------------------------------------------------------------ query-agnostic salience of an encoder layer
def _enc_case(seed, B=2, N=23, H=3, D=16):
    rng = np.random.default_rng(seed)
    f = lambda *s: rng.standard_normal(s).astype(np.float32)
    return f(B, N, H, D), f(B, H, N, D)


def test_salience_is_the_column_mean_of_library_attention_on_an_identity_value_matrix():
    """Library routine as a special case: SDPA (float64) with V = I returns the attention matrix itself;
    its column means over query tokens and heads are the salience."""
    q, k = _enc_case(11)
    B, N, H, D = q.shape
    sal, lse = oracle.salience_self(q, k)
    qt = torch.from_numpy(q.astype(np.float64)).permute(0, 2, 1, 3)      # [B, H, N, D]
    kt = torch.from_numpy(k.astype(np.float64))
    eye = torch.eye(N, dtype=torch.float64).expand(B, H, N, N)
    p = torch.nn.functional.scaled_dot_product_attention(qt, kt, eye).numpy()   # [B, H, query, key]
    assert np.allclose(sal, p.mean(axis=(1, 2)), rtol=1e-12, atol=1e-15)
    from scipy.special import logsumexp
    logits = np.einsum("bihd,bhjd->bihj", q.astype(np.float64), k.astype(np.float64)) / np.sqrt(D)
    assert np.allclose(lse, logsumexp(logits, axis=3), rtol=1e-12)


def test_salience_of_two_tokens_is_the_logistic_closed_form():
    """N = 2: a row's probability of key 0 is the logistic function of the logit difference; written with
    math.exp and plain loops.  Normalising over the wrong axis, or a transposed product, fails here."""
    import math
    q, k = _enc_case(12, B=1, N=2, H=2, D=8)
    sal, _ = oracle.salience_self(q, k)
    sc = 1.0 / math.sqrt(8)
    recv = [0.0, 0.0]
    for h in range(2):
        for i in range(2):
            l0 = sc * sum(float(q[0, i, h, d]) * float(k[0, h, 0, d]) for d in range(8))
            l1 = sc * sum(float(q[0, i, h, d]) * float(k[0, h, 1, d]) for d in range(8))
            p0 = 1.0 / (1.0 + math.exp(l1 - l0))
            recv[0] += p0
            recv[1] += 1.0 - p0
    assert np.allclose(sal[0], np.array(recv) / 4.0, rtol=1e-12)


def test_salience_with_one_shared_query_is_the_softmax_of_that_query():
    """Every token asks the same question, one head: all rows of the attention matrix are equal, so the
    salience is that row -- scipy's softmax of scale * K u.  Also fixes the explicit scale."""
    from scipy.special import softmax
    rng = np.random.default_rng(13)
    N, D = 31, 16
    u = rng.standard_normal(D).astype(np.float32)
    k = rng.standard_normal((1, 1, N, D)).astype(np.float32)
    q = np.broadcast_to(u, (1, N, 1, D)).copy()
    sal, _ = oracle.salience_self(q, k, scale=0.37)
    assert np.allclose(sal[0], softmax(0.37 * k[0, 0].astype(np.float64) @ u.astype(np.float64)), rtol=1e-12)


def test_salience_invariants():
    """Identical keys -> uniform 1/n; the salience of the live tokens sums to 1 for any lengths; adding a vector
    to every key changes nothing; permuting the tokens permutes the salience; permuting only who asks
    changes nothing; rows past vis_len are neither read nor counted."""
    q, k = _enc_case(14)
    B, N, H, D = q.shape
    k_same = np.broadcast_to(k[:, :, :1], k.shape).copy()
    sal, _ = oracle.salience_self(q, k_same)
    assert np.allclose(sal, 1.0 / N, rtol=1e-12)
    vis_len = np.array([N, 9], np.int32)
    sal, lse = oracle.salience_self(q, k, vis_len=vis_len)
    assert np.allclose([sal[0].sum(), sal[1, :9].sum()], 1.0, rtol=1e-12)
    assert np.all(np.isneginf(sal[1, 9:])) and np.all(np.isposinf(lse[1, 9:]))
    q2, k2 = q.copy(), k.copy()
    q2[1, 9:] = 1e4
    k2[1, :, 9:] = 1e4
    sal2, lse2 = oracle.salience_self(q2, k2, vis_len=vis_len)
    assert np.array_equal(sal2, sal) and np.array_equal(lse2, lse)
    full, _ = oracle.salience_self(q, k)
    shift = np.random.default_rng(15).standard_normal(D).astype(np.float32)
    moved, _ = oracle.salience_self(q.astype(np.float64), k.astype(np.float64) + shift)
    assert np.allclose(moved, full, rtol=1e-9)
    perm = np.random.default_rng(16).permutation(N)
    both, _ = oracle.salience_self(q[:, perm], k[:, :, perm])
    assert np.allclose(both, full[:, perm], rtol=1e-12)
    askers, _ = oracle.salience_self(q[:, perm], k)
    assert np.allclose(askers, full, rtol=1e-12)


def test_salience_of_a_dominant_key_approaches_one():
    """One key far along every query's direction takes all the attention."""
    rng = np.random.default_rng(17)
    N, D = 12, 8
    u = np.ones(D, np.float32)
    q = (np.abs(rng.standard_normal((1, N, 1, D))) + 0.5).astype(np.float32)   # positive along u
    k = rng.standard_normal((1, 1, N, D)).astype(np.float32)
    k[0, 0, 5] = 60.0 * u
    sal, _ = oracle.salience_self(q, k)
    assert sal[0, 5] > 1 - 1e-9 and np.all(sal[0, np.arange(N) != 5] < 1e-9)
