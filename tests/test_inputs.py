"""The seeded input generator: shapes, determinism, and the structure each config states."""
import numpy as np

import sv_inputs


def test_shapes_dtypes_and_determinism():
    for cfg in (1, 2):
        w = sv_inputs.workload(cfg)
        a, b = sv_inputs.make_inputs(w), sv_inputs.make_inputs(w)
        assert a["q"].shape == (w.B, w.n_q_heads, w.head_dim) and a["q"].dtype == w.np_dtype
        assert a["k_vis"].shape == (w.B, w.n_kv_heads, w.n_vis, w.head_dim)
        assert a["k_txt"].shape == (w.B, w.n_kv_heads, w.n_txt, w.head_dim)
        for key in a:
            assert np.array_equal(a[key], b[key])


def test_layers_fold_into_batch_with_their_own_seeds():
    w = sv_inputs.workload(3, n_vis=392, n_txt=16, k=39, layers=3)
    a = sv_inputs.make_inputs(w)
    assert a["k_vis"].shape[0] == 3
    one = sv_inputs.make_layer(w, 1)
    assert np.array_equal(a["k_vis"][1], one["k_vis"][0])
    assert not np.array_equal(a["k_vis"][0], a["k_vis"][1])


def test_planted_tokens_shift_five_percent_of_keys_along_the_summed_query():
    w = sv_inputs.workload(3, n_vis=2000, n_txt=16, k=200, layers=1)
    a = sv_inputs.make_layer(w, 0)
    base = sv_inputs.make_layer(sv_inputs.workload(3, n_vis=2000, n_txt=16, k=200, layers=1, structure="iid"), 0)
    diff = a["k_vis"].astype(np.float32) - base["k_vis"].astype(np.float32)
    moved = np.abs(diff).max(axis=-1) > 0.05
    assert np.all(moved.sum(axis=-1) == 100)
    G = 7
    for g in range(4):
        u = a["q"][0, g * G:(g + 1) * G].astype(np.float32).sum(0)
        u /= np.linalg.norm(u)
        proj = diff[0, g][moved[0, g]] @ u
        assert np.allclose(proj, 2.0, atol=0.05)


def test_frame_offsets_are_shared_inside_a_frame():
    w = sv_inputs.workload(4, n_vis=196 * 5, n_txt=8, k=49, layers=1)
    a = sv_inputs.make_layer(w, 0)
    base = sv_inputs.make_layer(sv_inputs.workload(4, n_vis=196 * 5, n_txt=8, k=49, layers=1, structure="iid"), 0)
    d = (a["k_vis"].astype(np.float32) - base["k_vis"].astype(np.float32))[0, 0].reshape(5, 196, 128)
    assert np.abs(d - d[:, :1]).max() < 0.02          # constant inside a frame (up to fp16 rounding)
    assert 0.3 < d[:, 0].std() < 0.7                  # offsets ~ N(0, 0.5^2)


def test_ragged_lengths_and_sentinel_padding():
    w = sv_inputs.workload(5)
    a = sv_inputs.make_inputs(w)
    vl = a["vis_len"]
    assert vl.shape == (16,) and vl.min() >= 4096 and vl.max() <= 8192
    for b in range(16):
        assert np.all(a["k_vis"][b, :, vl[b]:] == np.float16(sv_inputs.PAD_SENTINEL))
    q1 = sv_inputs.round_query(w, 1)
    assert q1.shape == a["q"].shape and not np.array_equal(q1, a["q"])


def test_algorithmic_bytes_of_the_long_video_config():
    w = sv_inputs.workload(4)
    vl = np.full(w.B, w.n_vis, np.int32)
    tl = np.full(w.B, w.n_txt, np.int32)
    assert sv_inputs.algorithmic_bytes(w, vl, tl) == 28 * 58_615_808
