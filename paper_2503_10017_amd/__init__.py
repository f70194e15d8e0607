"""MI355X-native fast reciprocal nearest-neighbour matching (the FastNN stage of Speedy MASt3R).

The work is done by hand-written HIP kernels behind the C ABI in ``include/fnn.h``
(``lib/libfnn.so``); this package only marshals torch tensors into that ABI.  There is
no CPU or eager fallback: calls raise if the library is missing.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    FNN_BF16,
    FNN_F16,
    FNN_F32,
    FnnError,
    fnn_mutual_dense,
    fnn_nearest,
    fnn_nearest_blocked,
    fnn_pairs_to_pixels,
    fnn_reciprocal,
    fnn_reciprocal_static,
    fnn_status_string,
    fnn_trace_begin,
    fnn_trace_end,
    fnn_measure_ceiling,
    fnn_workspace_bytes,
    fnn_workspace_bytes_opts,
    library_path,
    load_library,
)
