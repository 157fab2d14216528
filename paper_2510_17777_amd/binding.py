"""ctypes binding of the C ABI in include/sparsevila.h (argument marshalling only).

Every function here has the name and the argument order of its C entry point and
does nothing but turn torch device tensors into pointers.  All arithmetic runs in
the HIP kernels of libsparsevila.so.  PyTorch supplies device memory and streams.
"""
from __future__ import annotations

import contextlib
import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# SPARSEVILA_LIBRARY names another build of the same library to load instead (e.g. the host-sanitized one).
_LIB_PATH = os.environ.get("SPARSEVILA_LIBRARY") or os.path.join(_HERE, "libsparsevila.so")
_LIB_HOOKS_PATH = os.path.join(_HERE, "libsparsevila_hooks.so")
_lib: Optional[ctypes.CDLL] = None
_lib_hooks: Optional[ctypes.CDLL] = None

SV_F16, SV_F32 = 0, 1


class SVError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {sv_strerror(status)} (status {status})")


class SvShape(ctypes.Structure):
    """Mirror of struct sv_shape."""
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("n_vis_max", ctypes.c_int32), ("n_txt_max", ctypes.c_int32),
        ("k", ctypes.c_int32), ("dtype", ctypes.c_int32), ("scale", ctypes.c_float),
        ("reserved", ctypes.c_int32),
        ("vis_len", ctypes.c_void_p), ("txt_len", ctypes.c_void_p),
        ("q_stride_b", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
        ("kv_vis_stride_b", ctypes.c_int64), ("kv_vis_stride_h", ctypes.c_int64),
        ("kv_vis_stride_n", ctypes.c_int64),
        ("kv_txt_stride_b", ctypes.c_int64), ("kv_txt_stride_h", ctypes.c_int64),
        ("kv_txt_stride_n", ctypes.c_int64),
    ]


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Loads libsparsevila.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    _lib = _open(_LIB_PATH)
    return _lib


@contextlib.contextmanager
def test_hooks():
    """Inside the block every function of this module calls libsparsevila_hooks.so: the same kernel objects
    linked with a build of the C-ABI layer that knows two more knobs ("filter_test_mode", "step_stages"; see
    sv_has_test_hooks in the header).  For the repository's tests and benchmark only; the knobs are reset on exit."""
    global _lib, _lib_hooks
    if _lib_hooks is None:
        _lib_hooks = _open(_LIB_HOOKS_PATH)
        assert _lib_hooks.sv_has_test_hooks() == 1
    saved, _lib = _lib, _lib_hooks
    try:
        yield _lib_hooks
    finally:
        _lib_hooks.sv_set_tuning(b"filter_test_mode", 0)
        _lib_hooks.sv_set_tuning(b"step_stages", 3)
        _lib = saved


def _open(path: str) -> ctypes.CDLL:
    if not os.path.exists(path):
        raise RuntimeError(
            f"{path} is missing: build it with `python -m paper_2510_17777_amd.build` "
            "(hipcc, gfx950).  There is no CPU fallback for the sparse decode path.")
    lib = ctypes.CDLL(path)
    P, vp, i32, sz = ctypes.POINTER(SvShape), ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    lib.sv_shape_set_contiguous.restype = None
    lib.sv_shape_set_contiguous.argtypes = [P]
    lib.sv_workspace_bytes.restype = sz
    lib.sv_workspace_bytes.argtypes = [P]
    lib.sv_select_workspace_bytes.restype = sz
    lib.sv_select_workspace_bytes.argtypes = [P]
    lib.sv_score_visual.restype = ctypes.c_int
    lib.sv_score_visual.argtypes = [P, vp, vp, vp, vp]
    lib.sv_topk_select.restype = ctypes.c_int
    lib.sv_topk_select.argtypes = [P, vp, vp, vp, vp, sz, vp]
    lib.sv_sparse_decode_attn.restype = ctypes.c_int
    lib.sv_sparse_decode_attn.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.sv_decode_step.restype = ctypes.c_int
    lib.sv_decode_step.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.sv_decode_step_static.restype = ctypes.c_int
    lib.sv_decode_step_static.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.sv_mass_workspace_bytes.restype = sz
    lib.sv_mass_workspace_bytes.argtypes = [P, i32]
    lib.sv_score_visual_mass.restype = ctypes.c_int
    lib.sv_score_visual_mass.argtypes = [P, vp, i32, ctypes.c_int64, vp, vp, vp, vp, vp, sz, vp]
    lib.sv_salience_workspace_bytes.restype = sz
    lib.sv_salience_workspace_bytes.argtypes = [P]
    lib.sv_salience_self.restype = ctypes.c_int
    lib.sv_salience_self.argtypes = [P, vp, ctypes.c_int64, vp, vp, vp, vp, sz, vp]
    lib.sv_pack_selected.restype = ctypes.c_int
    lib.sv_pack_selected.argtypes = [P, vp, vp, vp, vp, vp, vp, vp]
    lib.sv_copy_bytes.restype = ctypes.c_int
    lib.sv_copy_bytes.argtypes = [vp, vp, sz, vp]
    lib.sv_read_bytes.restype = ctypes.c_int
    lib.sv_read_bytes.argtypes = [vp, sz, vp, vp]
    lib.sv_strerror.restype = ctypes.c_char_p
    lib.sv_strerror.argtypes = [ctypes.c_int]
    lib.sv_set_tuning.restype = ctypes.c_int
    lib.sv_set_tuning.argtypes = [ctypes.c_char_p, i32]
    lib.sv_get_tuning.restype = i32
    lib.sv_get_tuning.argtypes = [ctypes.c_char_p]
    lib.sv_has_test_hooks.restype = i32
    lib.sv_has_test_hooks.argtypes = []
    return lib


def sv_strerror(status: int) -> str:
    return load_library().sv_strerror(int(status)).decode()


def sv_set_tuning(name: str, value: int) -> None:
    st = load_library().sv_set_tuning(name.encode(), int(value))
    if st != 0:
        raise SVError(st, f"sv_set_tuning({name}, {value})")


def sv_get_tuning(name: str) -> int:
    return int(load_library().sv_get_tuning(name.encode()))


@dataclass
class Shape:
    """Keeps the ctypes struct together with the tensors its pointers refer to."""
    c: SvShape
    vis_len: Optional[torch.Tensor] = None
    txt_len: Optional[torch.Tensor] = None

    def __getattr__(self, name):
        return getattr(self.c, name)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("the sparse decode library takes device tensors only")
    return t.data_ptr()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float16:
        return SV_F16
    if t.dtype == torch.float32:
        return SV_F32
    raise TypeError(f"q/K/V must be float16 or float32, got {t.dtype}")


def _len_tensor(x, B: int, device) -> Optional[torch.Tensor]:
    if x is None:
        return None
    t = torch.as_tensor(x, dtype=torch.int32).to(device).contiguous()
    if t.shape != (B,):
        raise ValueError("length arrays must have shape [B]")
    return t


def make_shape(q: torch.Tensor, k_vis: torch.Tensor, k_txt: Optional[torch.Tensor], k: int,
               vis_len=None, txt_len=None, scale: float = 0.0) -> Shape:
    """Builds an sv_shape from the tensors' own sizes and strides.

    q [B,Hq,D]; k_vis [B,Hkv,Nv,D] (v_vis must share its strides); k_txt [B,Hkv,Nt,D] or None.
    """
    B, Hq, D = q.shape
    Bk, Hkv, Nv, Dk = k_vis.shape
    if (Bk, Dk) != (B, D):
        raise ValueError("q and k_vis disagree on batch or head_dim")
    if q.stride(2) != 1 or (Nv > 0 and k_vis.stride(3) != 1):
        raise ValueError("head_dim must be contiguous")
    s = SvShape()
    s.batch, s.n_q_heads, s.n_kv_heads, s.head_dim = B, Hq, Hkv, D
    s.n_vis_max, s.k, s.dtype, s.scale, s.reserved = Nv, int(k), _dtype_code(q), float(scale), 0
    s.q_stride_b, s.q_stride_h = q.stride(0), q.stride(1)
    s.kv_vis_stride_b, s.kv_vis_stride_h, s.kv_vis_stride_n = k_vis.stride(0), k_vis.stride(1), k_vis.stride(2)
    if k_txt is not None:
        if k_txt.shape[0] != B or k_txt.shape[1] != Hkv or k_txt.shape[3] != D:
            raise ValueError("k_txt disagrees with q/k_vis")
        s.n_txt_max = k_txt.shape[2]
        s.kv_txt_stride_b, s.kv_txt_stride_h, s.kv_txt_stride_n = k_txt.stride(0), k_txt.stride(1), k_txt.stride(2)
    else:
        s.n_txt_max = 0
        s.kv_txt_stride_b, s.kv_txt_stride_h, s.kv_txt_stride_n = 0, 0, D
    vl = _len_tensor(vis_len, B, q.device)
    tl = _len_tensor(txt_len, B, q.device)
    s.vis_len = _ptr(vl)
    s.txt_len = _ptr(tl)
    return Shape(s, vl, tl)


def workspace_bytes(shape: Shape) -> int:
    return int(load_library().sv_workspace_bytes(ctypes.byref(shape.c)))


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _check(st: int, where: str) -> None:
    if st != 0:
        raise SVError(st, where)


def _check_layout(shape: Shape, k_vis=None, v_vis=None, k_txt=None, v_txt=None) -> None:
    """The C ABI addresses K and V of a segment with ONE set of strides (the shape's): a tensor laid out
    differently would be read with the wrong strides, silently.  Compared here, where the tensors are known."""
    c = shape.c
    vis = (c.kv_vis_stride_b, c.kv_vis_stride_h, c.kv_vis_stride_n, 1)
    txt = (c.kv_txt_stride_b, c.kv_txt_stride_h, c.kv_txt_stride_n, 1)
    for name, t, rows, strides in (("k_vis", k_vis, c.n_vis_max, vis), ("v_vis", v_vis, c.n_vis_max, vis),
                                   ("k_txt", k_txt, c.n_txt_max, txt), ("v_txt", v_txt, c.n_txt_max, txt)):
        if t is None or rows == 0:
            continue
        if tuple(t.shape) != (c.batch, c.n_kv_heads, rows, c.head_dim):
            raise ValueError(f"{name} has shape {tuple(t.shape)}, the sv_shape says "
                             f"{(c.batch, c.n_kv_heads, rows, c.head_dim)}")
        # a dimension of size 1 has no meaningful stride
        if any(n > 1 and a != b for n, a, b in zip(t.shape, t.stride(), strides)):
            raise ValueError(f"{name} has strides {t.stride()}, the sv_shape says {strides}: K and V of a "
                             "segment must share one layout")
        if _dtype_code(t) != c.dtype:
            raise TypeError(f"{name} has dtype {t.dtype}, the sv_shape says code {c.dtype}")


def sv_score_visual(shape: Shape, q, k_vis, scores, stream=None) -> None:
    _check_layout(shape, k_vis=k_vis)
    _check(load_library().sv_score_visual(ctypes.byref(shape.c), _ptr(q), _ptr(k_vis), _ptr(scores),
                                          _stream(stream)), "sv_score_visual")


def sv_topk_select(shape: Shape, scores, idx, count, workspace=None, stream=None) -> None:
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().sv_topk_select(ctypes.byref(shape.c), _ptr(scores), _ptr(idx), _ptr(count),
                                         _ptr(workspace), nbytes, _stream(stream)), "sv_topk_select")


def sv_sparse_decode_attn(shape: Shape, q, k_vis, v_vis, k_txt, v_txt, idx, count, out, lse,
                          workspace, stream=None) -> None:
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check_layout(shape, k_vis, v_vis, k_txt, v_txt)
    _check(load_library().sv_sparse_decode_attn(
        ctypes.byref(shape.c), _ptr(q), _ptr(k_vis), _ptr(v_vis), _ptr(k_txt), _ptr(v_txt),
        _ptr(idx), _ptr(count), _ptr(out), _ptr(lse), _ptr(workspace), nbytes, _stream(stream)),
        "sv_sparse_decode_attn")


def sv_decode_step(shape: Shape, q, k_vis, v_vis, k_txt, v_txt, scores, idx, count, out, lse,
                   workspace, stream=None) -> None:
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check_layout(shape, k_vis, v_vis, k_txt, v_txt)
    _check(load_library().sv_decode_step(
        ctypes.byref(shape.c), _ptr(q), _ptr(k_vis), _ptr(v_vis), _ptr(k_txt), _ptr(v_txt),
        _ptr(scores), _ptr(idx), _ptr(count), _ptr(out), _ptr(lse), _ptr(workspace), nbytes,
        _stream(stream)), "sv_decode_step")


STATIC_SCRATCH_BYTES = 32 << 20


def sv_decode_step_static(shape: Shape, q, k_vis, v_vis, k_txt, v_txt, scores, idx, count, out, lse,
                          stream=None) -> None:
    """sv_decode_step without a workspace argument: the library's own per-GPU scratch array serves."""
    _check_layout(shape, k_vis, v_vis, k_txt, v_txt)
    _check(load_library().sv_decode_step_static(
        ctypes.byref(shape.c), _ptr(q), _ptr(k_vis), _ptr(v_vis), _ptr(k_txt), _ptr(v_txt),
        _ptr(scores), _ptr(idx), _ptr(count), _ptr(out), _ptr(lse), _stream(stream)), "sv_decode_step_static")


def sv_score_visual_mass(shape: Shape, q_multi, k_vis, k_txt, scores, lse=None, workspace=None, stream=None):
    """q_multi [B, Tq, Hq, D] (any strides with D contiguous); shape built from q_multi[:, 0]."""
    Tq = q_multi.shape[1]
    if (shape.c.q_stride_b, shape.c.q_stride_h) != (q_multi.stride(0), q_multi.stride(2)):
        raise ValueError("the shape's query strides do not describe q_multi: build it from q_multi[:, 0]")
    if workspace is None:
        nbytes = int(load_library().sv_mass_workspace_bytes(ctypes.byref(shape.c), Tq))
        workspace = torch.empty((max(nbytes, 256),), dtype=torch.uint8, device=q_multi.device)
    _check(load_library().sv_score_visual_mass(
        ctypes.byref(shape.c), _ptr(q_multi), Tq, q_multi.stride(1), _ptr(k_vis), _ptr(k_txt), _ptr(scores),
        _ptr(lse), _ptr(workspace), workspace.numel(), _stream(stream)), "sv_score_visual_mass")
    return workspace


def make_encoder_shape(q_all: torch.Tensor, k_all: torch.Tensor, vis_len=None, scale: float = 0.0) -> Shape:
    """sv_shape of one encoder layer for sv_salience_self: q_all [B, N, H, D], k_all [B, H, N, D] (any strides
    with D contiguous; views of a fused qkv tensor are fine)."""
    B, N, H, D = q_all.shape
    if tuple(k_all.shape) != (B, H, N, D):
        raise ValueError("k_all must be [B, H, N, D] for q_all [B, N, H, D]")
    if q_all.stride(3) != 1 or k_all.stride(3) != 1:
        raise ValueError("head_dim must be contiguous")
    s = SvShape()
    s.batch, s.n_q_heads, s.n_kv_heads, s.head_dim = B, H, H, D
    s.n_vis_max, s.n_txt_max, s.k, s.dtype, s.scale, s.reserved = N, 0, 0, _dtype_code(q_all), float(scale), 0
    s.q_stride_b, s.q_stride_h = q_all.stride(0), q_all.stride(2)
    s.kv_vis_stride_b, s.kv_vis_stride_h, s.kv_vis_stride_n = k_all.stride(0), k_all.stride(1), k_all.stride(2)
    s.kv_txt_stride_b, s.kv_txt_stride_h, s.kv_txt_stride_n = 0, 0, D
    vl = _len_tensor(vis_len, B, q_all.device)
    s.vis_len = _ptr(vl)
    s.txt_len = None
    return Shape(s, vl, None)


def sv_salience_self(shape: Shape, q_all, k_all, salience, lse=None, workspace=None, stream=None):
    """shape from make_encoder_shape; salience [B, N] fp32; returns the workspace it used."""
    if (shape.c.q_stride_b, shape.c.q_stride_h) != (q_all.stride(0), q_all.stride(2)) or \
            (shape.c.kv_vis_stride_b, shape.c.kv_vis_stride_h, shape.c.kv_vis_stride_n) != k_all.stride()[:3]:
        raise ValueError("the shape's strides do not describe q_all / k_all: build it with make_encoder_shape")
    if workspace is None:
        nbytes = int(load_library().sv_salience_workspace_bytes(ctypes.byref(shape.c)))
        workspace = torch.empty((max(nbytes, 256),), dtype=torch.uint8, device=q_all.device)
    _check(load_library().sv_salience_self(
        ctypes.byref(shape.c), _ptr(q_all), q_all.stride(1), _ptr(k_all), _ptr(salience), _ptr(lse),
        _ptr(workspace), workspace.numel(), _stream(stream)), "sv_salience_self")
    return workspace


def sv_pack_selected(shape: Shape, k_vis, v_vis, idx, count, k_pack, v_pack, stream=None) -> None:
    _check_layout(shape, k_vis, v_vis)
    c = shape.c
    for name, t in (("k_pack", k_pack), ("v_pack", v_pack)):
        if c.k > 0 and (tuple(t.shape) != (c.batch, c.n_kv_heads, c.k, c.head_dim) or not t.is_contiguous()):
            raise ValueError(f"{name} must be a dense [B, Hkv, k, D] tensor")
    _check(load_library().sv_pack_selected(ctypes.byref(shape.c), _ptr(k_vis), _ptr(v_vis), _ptr(idx), _ptr(count),
                                           _ptr(k_pack), _ptr(v_pack), _stream(stream)), "sv_pack_selected")


def sv_copy_bytes(dst: torch.Tensor, src: torch.Tensor, nbytes: int, stream=None) -> None:
    _check(load_library().sv_copy_bytes(_ptr(dst), _ptr(src), int(nbytes), _stream(stream)), "sv_copy_bytes")


READ_SINK_BYTES = 4096


def sv_read_bytes(src: torch.Tensor, nbytes: int, sink: torch.Tensor, stream=None) -> None:
    """Plain read stream over nbytes of src (measurement aid); sink: READ_SINK_BYTES bytes on the device."""
    if sink.numel() * sink.element_size() < READ_SINK_BYTES:
        raise ValueError("sink too small")
    _check(load_library().sv_read_bytes(_ptr(src), int(nbytes), _ptr(sink), _stream(stream)), "sv_read_bytes")


class DecodeBuffers:
    """Output and workspace tensors of one shape, allocated once through torch."""

    def __init__(self, shape: Shape, device, with_scores: bool = True):
        s = shape.c
        B, Hq, Hkv, D = s.batch, s.n_q_heads, s.n_kv_heads, s.head_dim
        self.scores = torch.empty((B, Hkv, s.n_vis_max), dtype=torch.float32, device=device) if with_scores else None
        self.idx = torch.empty((B, Hkv, s.k), dtype=torch.int32, device=device)
        self.count = torch.empty((B, Hkv), dtype=torch.int32, device=device)
        self.out = torch.empty((B, Hq, D), dtype=torch.float32, device=device)
        self.lse = torch.empty((B, Hq), dtype=torch.float32, device=device)
        nbytes = workspace_bytes(shape)
        if nbytes == 0:
            raise SVError(-2, "sv_workspace_bytes")
        self.workspace = torch.empty((nbytes,), dtype=torch.uint8, device=device)
