"""MI355X-native sparse frame-difference CNN inference (DeltaCNN's hot path).

The work is done by hand-written HIP kernels for gfx950 in `lib/libdeltacnn.so` (C ABI in
`include/deltacnn.h`); this package only marshals arguments.  Build the library with
`python -m paper_2203_03996_amd.build` (or `__graft_entry__.build()`).
"""
from .binding import (  # noqa: F401
    ACCUM, ACT, CONCAT, GAVGPOOL, UPSAMPLE_BILINEAR, ACT_CODES, ACT_NONE, ACT_RELU, ACT_RELU6, CONV, DELTAGEN, DWCONV, F16, F32, MAXPOOL, UPSAMPLE,
    Context, DcnnError, Delta, Layer, Net, EXPORTS, LIB_PATH, load_library, make_desc,
)
