"""MI355X-native large-model support: graph rewriting with swap-out / swap-in operations and a
budgeted executor with gfx950 convolution kernels, behind the C ABI of include/lms.h.

This package is a thin binding: argument marshalling only, every step of the path runs inside
liblms.so.  Import fails to do any work unless the library has been built
(`python -m paper_1807_02037_amd.build`).
"""
from . import _lib as abi  # noqa: F401
from .api import (  # noqa: F401
    LmsError, Graph, Executor, params, conv_fwd, conv_dgrad, conv_wgrad, conv_wgrad_bias, conv_wgrad_static, static_scratch_bytes, swap_staging_bytes, swap_encode_staged, swap_decode_staged, conv_workspace_bytes, conv_desc,
    swap_encoded_bytes, swap_encode, swap_decode, swap_moved_bytes,
)
from .models import build_graph  # noqa: F401
