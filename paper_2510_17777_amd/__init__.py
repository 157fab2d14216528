"""MI355X (gfx950) sparse decode path of SparseVILA: score -> top-k -> sparse attention.

The package is a thin ctypes binding over ``libsparsevila.so`` (hand-written HIP
kernels behind the C ABI declared in ``include/sparsevila.h``).  There is no CPU
fallback: calling any entry point without the built library raises.
"""
from .binding import (  # noqa: F401
    SVError, SvShape, Shape, library_path, load_library, make_shape, workspace_bytes,
    sv_score_visual, sv_topk_select, sv_sparse_decode_attn, sv_decode_step, sv_decode_step_static,
    STATIC_SCRATCH_BYTES,
    sv_pack_selected, sv_score_visual_mass, sv_salience_self, make_encoder_shape, sv_set_tuning, sv_get_tuning,
    sv_strerror, test_hooks, sv_copy_bytes, sv_read_bytes, READ_SINK_BYTES, DecodeBuffers,
)
