"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and
rejects bad arguments on the host before anything could be launched (no GPU needed:
none of these calls gets as far as a kernel launch)."""
import ctypes
import os
import re

import pytest

import paper_2510_17777_amd as sv
from paper_2510_17777_amd.binding import SvShape

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sparsevila.h")

OK, E_NULL, E_SHAPE, E_DTYPE, E_ALIGN, E_WS, E_LAUNCH = 0, -1, -2, -3, -4, -5, -6
FAKE = 0x7F0000001000      # never dereferenced by the host code under test (4 KiB aligned)


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sv_[a-z_]+)\s*\(", text)))


def good_shape(**kw) -> SvShape:
    s = SvShape()
    s.batch, s.n_q_heads, s.n_kv_heads, s.head_dim = 2, 28, 4, 128
    s.n_vis_max, s.n_txt_max, s.k, s.dtype, s.scale, s.reserved = 1000, 64, 100, 0, 0.0, 0
    for key, val in kw.items():
        setattr(s, key, val)
    sv.load_library().sv_shape_set_contiguous(ctypes.byref(s))
    return s


def test_header_declares_the_expected_entry_points():
    names = declared_functions()
    for must in ("sv_score_visual", "sv_topk_select", "sv_sparse_decode_attn", "sv_decode_step",
                 "sv_pack_selected", "sv_score_visual_mass", "sv_mass_workspace_bytes", "sv_salience_self", "sv_salience_workspace_bytes", "sv_workspace_bytes", "sv_strerror", "sv_shape_set_contiguous"):
        assert must in names


def test_library_exports_every_declared_symbol():
    lib = sv.load_library()
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in sparsevila.h but not exported"


def test_struct_layout_matches_the_header():
    # 10 4-byte fields, 2 pointers, 8 int64 strides
    assert ctypes.sizeof(SvShape) == 10 * 4 + 2 * 8 + 8 * 8
    assert SvShape.vis_len.offset == 40 and SvShape.q_stride_b.offset == 56


def test_contiguous_strides():
    s = good_shape()
    assert (s.q_stride_h, s.q_stride_b) == (128, 128 * 28)
    assert (s.kv_vis_stride_n, s.kv_vis_stride_h, s.kv_vis_stride_b) == (128, 128000, 512000)
    assert (s.kv_txt_stride_n, s.kv_txt_stride_h, s.kv_txt_stride_b) == (128, 8192, 32768)


def test_workspace_size_is_positive_aligned_and_monotone():
    lib = sv.load_library()
    a = lib.sv_workspace_bytes(ctypes.byref(good_shape()))
    b = lib.sv_workspace_bytes(ctypes.byref(good_shape(n_vis_max=2000)))
    c = lib.sv_workspace_bytes(ctypes.byref(good_shape(k=900)))
    assert a > 0 and a % 256 == 0 and b > a and c > a
    # scores + partial accumulators + partial (max, sum) for 64-token chunks
    S = (64 + 100 + 63) // 64
    assert a >= 2 * 4 * 1000 * 4 + 2 * 28 * S * (128 + 2) * 4
    assert lib.sv_workspace_bytes(ctypes.byref(good_shape(head_dim=96))) == 0
    assert lib.sv_workspace_bytes(None) == 0


@pytest.mark.parametrize("field,value,want", [
    ("batch", 0, E_SHAPE), ("batch", 70000, E_SHAPE), ("n_kv_heads", 0, E_SHAPE),
    ("n_q_heads", 30, E_SHAPE), ("head_dim", 96, E_SHAPE), ("n_vis_max", -1, E_SHAPE),
    ("n_txt_max", -1, E_SHAPE), ("k", -1, E_SHAPE), ("dtype", 2, E_DTYPE),
    ("scale", -1.0, E_SHAPE), ("scale", float("nan"), E_SHAPE), ("reserved", 1, E_SHAPE),
])
def test_bad_shape_fields_are_rejected(field, value, want):
    lib = sv.load_library()
    s = good_shape()
    setattr(s, field, value)
    assert lib.sv_score_visual(ctypes.byref(s), FAKE, FAKE, FAKE, None) == want
    assert lib.sv_decode_step(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                              None, FAKE, 1 << 40, None) == want


def test_strides_are_checked():
    lib = sv.load_library()
    s = good_shape()
    s.kv_vis_stride_n = 64                 # rows would overlap
    assert lib.sv_score_visual(ctypes.byref(s), FAKE, FAKE, FAKE, None) == E_SHAPE
    s = good_shape()
    s.kv_vis_stride_n = 132                # 264-byte rows: not a multiple of 16
    assert lib.sv_score_visual(ctypes.byref(s), FAKE, FAKE, FAKE, None) == E_ALIGN
    s = good_shape()
    s.q_stride_h = 129
    assert lib.sv_score_visual(ctypes.byref(s), FAKE, FAKE, FAKE, None) == E_ALIGN
    s = good_shape()
    s.kv_txt_stride_h = 4
    assert lib.sv_sparse_decode_attn(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                                     None, FAKE, 1 << 40, None) == E_ALIGN


def test_null_and_misaligned_pointers_are_rejected():
    lib = sv.load_library()
    s = good_shape()
    sp = ctypes.byref(s)
    assert lib.sv_score_visual(None, FAKE, FAKE, FAKE, None) == E_NULL
    assert lib.sv_score_visual(sp, None, FAKE, FAKE, None) == E_NULL
    assert lib.sv_score_visual(sp, FAKE, None, FAKE, None) == E_NULL
    assert lib.sv_score_visual(sp, FAKE, FAKE, None, None) == E_NULL
    assert lib.sv_score_visual(sp, FAKE + 8, FAKE, FAKE, None) == E_ALIGN
    assert lib.sv_score_visual(sp, FAKE, FAKE + 2, FAKE, None) == E_ALIGN
    assert lib.sv_topk_select(sp, FAKE, None, FAKE, None, 0, None) == E_NULL
    assert lib.sv_topk_select(sp, FAKE, FAKE, None, None, 0, None) == E_NULL
    assert lib.sv_topk_select(sp, None, FAKE, FAKE, None, 0, None) == E_NULL
    args = [FAKE] * 9
    for missing in (0, 1, 2, 3, 4, 6, 7):             # q, k_vis, v_vis, k_txt, v_txt, (idx: NULL = packed), count, out
        a = list(args)
        a[missing] = None
        a[8] = None                                    # lse is optional
        assert lib.sv_sparse_decode_attn(sp, *a, FAKE, 1 << 40, None) == E_NULL, missing
    a = [FAKE] * 8 + [None]
    a[2] = FAKE + 4
    assert lib.sv_sparse_decode_attn(sp, *a, FAKE, 1 << 40, None) == E_ALIGN
    pk = [FAKE] * 6                                    # k_vis, v_vis, idx, count, k_pack, v_pack
    for missing in range(6):
        a = list(pk)
        a[missing] = None
        assert lib.sv_pack_selected(sp, *a, None) == E_NULL, missing
    a = list(pk)
    a[4] = FAKE + 8
    assert lib.sv_pack_selected(sp, *a, None) == E_ALIGN


def test_workspace_is_checked():
    lib = sv.load_library()
    s = good_shape()
    sp = ctypes.byref(s)
    need = lib.sv_workspace_bytes(sp)
    a = [FAKE] * 8 + [None]
    assert lib.sv_sparse_decode_attn(sp, *a, None, need, None) == E_WS
    assert lib.sv_sparse_decode_attn(sp, *a, FAKE, need - 1, None) == E_WS
    assert lib.sv_sparse_decode_attn(sp, *a, FAKE + 128, need, None) == E_WS
    d = [FAKE] * 10
    assert lib.sv_decode_step(sp, *d, FAKE, need - 1, None) == E_WS


def test_text_only_shape_needs_no_visual_pointers():
    lib = sv.load_library()
    s = good_shape(k=0)
    sp = ctypes.byref(s)
    # k == 0: k_vis/v_vis/idx/count may be NULL; the call gets past validation, and what
    # happens next depends on the presence of a GPU, so only the workspace error is probed.
    assert lib.sv_sparse_decode_attn(sp, FAKE, None, None, FAKE, FAKE, None, None, FAKE, None,
                                     None, 0, None) == E_WS


def test_strerror_and_tuning_knobs():
    assert sv.sv_strerror(0) == "ok"
    for code in range(-6, 0):
        assert sv.sv_strerror(code) not in ("ok", "unknown status")
    assert sv.sv_strerror(-99) == "unknown status"
    lib = sv.load_library()
    assert sv.sv_get_tuning("attn_chunk") >= 64
    assert lib.sv_set_tuning(b"attn_chunk", 100) == E_SHAPE        # not a multiple of 64
    assert lib.sv_set_tuning(b"attn_chunk", 4096) == E_SHAPE
    assert lib.sv_set_tuning(b"score_rows_per_block", 8) == E_SHAPE
    assert lib.sv_set_tuning(b"no_such_knob", 1) == E_SHAPE
    assert lib.sv_set_tuning(None, 1) == E_NULL
    before = sv.sv_get_tuning("attn_chunk")
    sv.sv_set_tuning("attn_chunk", 256)
    assert sv.sv_get_tuning("attn_chunk") == 256
    sv.sv_set_tuning("attn_chunk", 0)
    assert sv.sv_get_tuning("attn_chunk") == before
    assert sv.sv_get_tuning("attn_batches") == 0                    # planned per call
    assert lib.sv_set_tuning(b"attn_batches", 9) == E_SHAPE
    assert lib.sv_set_tuning(b"attn_batches", -1) == E_SHAPE
    sv.sv_set_tuning("attn_batches", 5)
    assert sv.sv_get_tuning("attn_batches") == 5
    sv.sv_set_tuning("attn_batches", 0)


def test_product_library_has_no_test_hooks_and_the_test_build_exports_the_same_abi():
    """libsparsevila.so knows no knob that can leave an output unwritten or falsify a kernel's behaviour; the
    test build (same kernel objects, -DSV_TEST_HOOKS in the C-ABI layer) adds exactly those two names."""
    lib = sv.load_library()
    assert lib.sv_has_test_hooks() == 0
    for name in (b"filter_test_mode", b"step_stages"):
        assert lib.sv_set_tuning(name, 1) == E_SHAPE
        assert lib.sv_get_tuning(name) == -1
    with sv.test_hooks() as hooks:
        assert hooks is not lib and hooks.sv_has_test_hooks() == 1
        assert sv.load_library() is hooks                      # inside the block the binding calls the test build
        for name in declared_functions():
            assert hasattr(hooks, name), name
        assert hooks.sv_set_tuning(b"step_stages", 1) == OK and hooks.sv_get_tuning(b"step_stages") == 1
        assert hooks.sv_set_tuning(b"step_stages", 0) == E_SHAPE and hooks.sv_set_tuning(b"step_stages", 4) == E_SHAPE
        assert hooks.sv_set_tuning(b"filter_test_mode", 2) == OK
        assert hooks.sv_set_tuning(b"filter_test_mode", 3) == E_SHAPE
        assert lib.sv_get_tuning(b"step_stages") == -1         # the product's state is its own
    assert sv.load_library() is lib
    assert hooks.sv_get_tuning(b"step_stages") == 3 and hooks.sv_get_tuning(b"filter_test_mode") == 0   # reset on exit


def test_knobs_are_atomic_words_that_concurrent_setters_cannot_tear():
    """Each knob is one atomic word: threads hammering sv_set_tuning with valid values while others read leave
    every read a value that some thread wrote."""
    import threading
    lib = sv.load_library()
    seen, stop = set(), threading.Event()

    def setter(v):
        while not stop.is_set():
            assert lib.sv_set_tuning(b"attn_batches", v) == OK

    def reader():
        for _ in range(20000):
            seen.add(lib.sv_get_tuning(b"attn_batches"))

    threads = [threading.Thread(target=setter, args=(v,)) for v in (1, 8)] + [threading.Thread(target=reader)]
    for t in threads:
        t.start()
    threads[-1].join()
    stop.set()
    for t in threads[:-1]:
        t.join()
    lib.sv_set_tuning(b"attn_batches", 0)
    assert seen <= {0, 1, 8}


def test_select_workspace_depends_on_the_fields_the_selection_reads_only():
    """sv_topk_select reads batch, n_kv_heads, n_vis_max, vis_len and k: the workspace it asks for must not change
    with dtype, head_dim, the query heads or the text fields, and sv_workspace_bytes covers it."""
    lib = sv.load_library()

    def need(**kw):
        s = good_shape(**dict(dict(batch=2, n_kv_heads=2, n_q_heads=2, n_vis_max=60000, k=3000), **kw))
        sp = ctypes.byref(s)
        n = lib.sv_select_workspace_bytes(sp)
        assert 0 < n <= lib.sv_workspace_bytes(sp) and n % 256 == 0
        assert lib.sv_topk_select(sp, FAKE, FAKE, FAKE, None, 0, None) == E_WS          # long rows need one
        assert lib.sv_topk_select(sp, FAKE, FAKE, FAKE, FAKE, n - 256, None) == E_WS    # one granule short
        assert lib.sv_topk_select(sp, FAKE, FAKE, FAKE, FAKE + 16, n, None) == E_WS     # misaligned
        return n

    base = need()
    for kw in (dict(dtype=1), dict(head_dim=64), dict(n_q_heads=14), dict(n_txt_max=4096), dict(dtype=1, head_dim=64)):
        assert need(**kw) == base, kw
    assert need(n_vis_max=120000) > base and need(batch=4) > base
    short = good_shape(n_vis_max=16384, k=100)
    assert lib.sv_select_workspace_bytes(ctypes.byref(short)) == 0                       # selected on chip
    assert lib.sv_select_workspace_bytes(ctypes.byref(good_shape(head_dim=100))) == 0    # invalid shape


def test_measurement_aids_check_their_arguments():
    lib = sv.load_library()
    lib.sv_read_bytes.restype = ctypes.c_int
    lib.sv_read_bytes.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.sv_read_bytes(None, 1024, 4096, None) == E_NULL
    assert lib.sv_read_bytes(4096, 1024, None, None) == E_NULL
    assert lib.sv_read_bytes(4096, 1000, 8192, None) == E_ALIGN     # not a multiple of 16
    assert lib.sv_read_bytes(4100, 1024, 8192, None) == E_ALIGN
    assert lib.sv_copy_bytes(None, 4096, 1024, None) == E_NULL
    assert lib.sv_copy_bytes(4096, 8192, 1001, None) == E_ALIGN


def test_binding_refuses_host_tensors():
    import torch
    q = torch.zeros((1, 4, 64), dtype=torch.float16)
    k = torch.zeros((1, 1, 8, 64), dtype=torch.float16)
    shape = sv.make_shape(q, k, None, 2)
    with pytest.raises(ValueError):
        sv.sv_score_visual(shape, q, k, torch.zeros((1, 1, 8)))


def test_binding_refuses_value_tensors_laid_out_differently_from_the_keys():
    """K and V of a segment share the shape's strides: a V tensor in another layout (or of another size or
    dtype) would be read with K's strides, so the binding refuses it before any pointer is taken."""
    import torch
    B, Hq, Hkv, D, Nv, Nt = 2, 4, 2, 64, 24, 8
    q = torch.zeros((B, Hq, D), dtype=torch.float16)
    k_vis = torch.zeros((B, Hkv, Nv, D), dtype=torch.float16)
    k_txt = torch.zeros((B, Hkv, Nt, D), dtype=torch.float16)
    shape = sv.make_shape(q, k_vis, k_txt, 4)
    token_major = torch.zeros((B, Nv, Hkv, D), dtype=torch.float16).permute(0, 2, 1, 3)     # same sizes, other strides
    args = dict(idx=None, count=None, out=None, lse=None, workspace=None)
    with pytest.raises(ValueError, match="strides"):
        sv.sv_sparse_decode_attn(shape, q, k_vis, token_major, k_txt, k_txt, **args)
    with pytest.raises(ValueError, match="strides"):
        sv.sv_decode_step(shape, q, k_vis, k_vis, k_txt, torch.zeros((B, Nt, Hkv, D), dtype=torch.float16).permute(0, 2, 1, 3),
                          None, None, None, None, None, None)
    with pytest.raises(ValueError, match="shape"):
        sv.sv_sparse_decode_attn(shape, q, k_vis, k_vis[:, :, :-1], k_txt, k_txt, **args)
    with pytest.raises(TypeError):
        sv.sv_sparse_decode_attn(shape, q, k_vis, k_vis.float(), k_txt, k_txt, **args)
    with pytest.raises(ValueError, match="strides"):
        sv.sv_pack_selected(shape, k_vis, token_major, None, None, None, None)
    with pytest.raises(ValueError, match="device"):         # matching layouts get as far as the pointer check
        sv.sv_sparse_decode_attn(shape, q, k_vis, k_vis.clone(), k_txt, k_txt.clone(), **args)


def test_static_scratch_entry_point_checks_arguments_and_size_on_the_host():
    """sv_decode_step_static validates like sv_decode_step and rejects a shape whose scratch exceeds the
    library's array before anything touches a device (so this runs without a GPU)."""
    lib = sv.load_library()
    s = good_shape()
    sp = ctypes.byref(s)
    assert lib.sv_workspace_bytes(sp) <= sv.STATIC_SCRATCH_BYTES
    d = [FAKE] * 5
    assert lib.sv_decode_step_static(None, *d, FAKE, FAKE, FAKE, FAKE, FAKE, None) == E_NULL
    assert lib.sv_decode_step_static(sp, None, *d[1:], FAKE, FAKE, FAKE, FAKE, FAKE, None) == E_NULL
    assert lib.sv_decode_step_static(sp, *d, FAKE, None, FAKE, FAKE, FAKE, None) == E_NULL      # idx with k > 0
    assert lib.sv_decode_step_static(sp, *d, FAKE, FAKE, FAKE, None, FAKE, None) == E_NULL      # out
    assert lib.sv_decode_step_static(sp, FAKE + 8, *d[1:], FAKE, FAKE, FAKE, FAKE, FAKE, None) == E_ALIGN
    bad = good_shape(head_dim=100)
    assert lib.sv_decode_step_static(ctypes.byref(bad), *d, FAKE, FAKE, FAKE, FAKE, FAKE, None) == E_SHAPE
    # the long video with all 28 layers folded into the batch needs more than the array holds
    big = good_shape(batch=28, n_vis_max=50176, n_txt_max=1024, k=2509)
    assert lib.sv_workspace_bytes(ctypes.byref(big)) > sv.STATIC_SCRATCH_BYTES
    assert lib.sv_decode_step_static(ctypes.byref(big), *d, FAKE, FAKE, FAKE, FAKE, FAKE, None) == E_WS
    # what the header promises to fit
    for kw in (dict(batch=8, n_vis_max=50176, n_txt_max=1024, k=2509), dict(batch=28, n_vis_max=12544, n_txt_max=512, k=1254),
               dict(batch=16, n_vis_max=8192, n_txt_max=1024, k=512)):
        assert 0 < lib.sv_workspace_bytes(ctypes.byref(good_shape(**kw))) <= sv.STATIC_SCRATCH_BYTES, kw


def test_salience_entry_point_checks_its_arguments():
    lib = sv.load_library()
    s = good_shape(n_q_heads=16, n_kv_heads=16, head_dim=96, n_vis_max=5000)
    sp = ctypes.byref(s)
    need = lib.sv_salience_workspace_bytes(sp)
    assert need > 0 and need % 256 == 0
    ok_args = (FAKE, 16 * 96, FAKE, FAKE, None)          # q_all, q_stride_t, k_all, salience, lse (optional)
    assert lib.sv_salience_self(sp, *ok_args, FAKE, need - 1, None) == E_WS
    assert lib.sv_salience_self(sp, *ok_args, None, need, None) == E_WS
    assert lib.sv_salience_self(sp, None, 16 * 96, FAKE, FAKE, None, FAKE, need, None) == E_NULL
    assert lib.sv_salience_self(sp, FAKE, 16 * 96, None, FAKE, None, FAKE, need, None) == E_NULL
    assert lib.sv_salience_self(sp, FAKE, 16 * 96, FAKE, None, None, FAKE, need, None) == E_NULL
    assert lib.sv_salience_self(sp, FAKE + 8, 16 * 96, FAKE, FAKE, None, FAKE, need, None) == E_ALIGN
    assert lib.sv_salience_self(sp, FAKE, 16 * 96 + 4, FAKE, FAKE, None, FAKE, need, None) == E_ALIGN
    assert lib.sv_salience_self(sp, FAKE, 64, FAKE, FAKE, None, FAKE, need, None) == E_SHAPE      # token stride < D
    for bad, want in ((dict(n_q_heads=32), E_SHAPE),      # grouped heads: an encoder layer has none
                      (dict(head_dim=72), E_SHAPE),       # pad to 96
                      (dict(dtype=1), E_DTYPE),
                      (dict(batch=0), E_SHAPE)):
        t = good_shape(**{**dict(n_q_heads=16, n_kv_heads=16, head_dim=96, n_vis_max=5000), **bad})
        assert lib.sv_salience_workspace_bytes(ctypes.byref(t)) == 0
        assert lib.sv_salience_self(ctypes.byref(t), *ok_args, FAKE, 1 << 40, None) == want, bad
    # the other entry points still refuse head_dim 96
    assert lib.sv_workspace_bytes(sp) == 0
    # an empty layer does nothing and needs nothing
    e = good_shape(n_q_heads=16, n_kv_heads=16, head_dim=64, n_vis_max=0)
    assert lib.sv_salience_self(ctypes.byref(e), None, 16 * 64, None, None, None, None, 0, None) == OK
    # the workspace grows with the layer
    big = good_shape(n_q_heads=16, n_kv_heads=16, head_dim=96, n_vis_max=20000)
    assert lib.sv_salience_workspace_bytes(ctypes.byref(big)) > need


def test_head_dim_96_is_for_the_two_attention_mass_calls_only():
    lib = sv.load_library()
    s = good_shape(head_dim=96)
    sp = ctypes.byref(s)
    assert lib.sv_mass_workspace_bytes(sp, 8) > 0
    assert lib.sv_score_visual_mass(sp, FAKE, 8, 28 * 96, FAKE, FAKE, FAKE, None, FAKE, 16, None) == E_WS   # past the shape check
    assert lib.sv_workspace_bytes(sp) == 0
    assert lib.sv_score_visual(sp, FAKE, FAKE, FAKE, None) == E_SHAPE
    assert lib.sv_decode_step(sp, *([FAKE] * 10), FAKE, 1 << 40, None) == E_SHAPE
