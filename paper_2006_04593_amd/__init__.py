"""MI355X-native batched function-secret-sharing KeyGen / Eval (AriaNN, arXiv 2006.04593).

The work happens in libfss_mi355.so (hand-written HIP for gfx950 behind the C ABI of
include/fss.h); this package only marshals arguments.  There is no CPU fallback: if the
library has not been built, importing `binding` functions raises.
"""
from .binding import (  # noqa: F401
    argmax_count_mask,
    argmax_diff_mask,
    dot_finish,
    eq_mask,
    eq_masked_eval,
    maxpool_unroll,
    mul_open,
    FssError,
    build,
    clock_probe,
    cmp_chunked_key_bytes,
    cmp_eval,
    cmp_eval_streamed,
    cmp_eval_streamed_static,
    static_staging_bytes,
    wall_clock_khz,
    cmp_gen,
    cmp_key_bytes,
    eq_eval,
    eq_gen,
    eq_key_bytes,
    lib,
    library_path,
    prepare,
    quad_layout_below,
    relu_finish,
    relu_open,
    sign_eval,
    sign_mask,
)
