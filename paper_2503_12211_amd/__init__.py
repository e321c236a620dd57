"""Strassen-Tile (STL) operator for AMD MI355X: thin Python binding over the C-ABI HIP library.

Everything numerical happens in ``libstl_mi355x.so`` (hand-written gfx950 kernels).  This
package only marshals arguments; it has no CPU or PyTorch fallback and raises if the
library has not been built (``python -m paper_2503_12211_amd.build``).
"""
from .binding import (  # noqa: F401
    STL_BF16, STL_F32, STL_FLAG_AUTO, STL_FLAG_B_TRANSPOSED, STL_FLAG_EPILOGUE, STL_FLAG_FUSED, STL_FLAG_GELU, STL_FLAG_PIPELINED, STL_FLAG_UNFUSED,
    STL_OP_BACKWARD, STL_PLANE_GROUP, STL_OP_ENCODE_WEIGHT, STL_OP_ENCODE_WEIGHT_BACKWARD, STL_OP_FORWARD, Problem, StlError, exported_symbols, library_path,
    stl_aa_backward, stl_aa_forward, stl_aa_workspace_bytes, stl_backward, stl_decode, stl_encode_activation, stl_encode_weight, stl_encode_weight_backward, stl_forward, stl_forward_static, STL_STATIC_SCRATCH_BYTES, stl_last_error,
    stl_mlp_forward, stl_mlp_workspace_bytes, stl_plane_elems, stl_plane_matmul, stl_ragged_backward, stl_ragged_forward, stl_ragged_workspace_bytes, stl_recode, stl_status_string, stl_version,
    stl_workspace_bytes,
)
