"""MI355X (gfx950) implementation of the Sparse VideoGen2 sparse-attention layer path.

The product is the C-ABI library `libsvg2_hip.so` (see include/svg2.h); this
package holds its HIP sources (csrc/), the build step (build.py), a ctypes
binding with the same entry-point names (binding.py) and the synthetic input
generators (workloads.py).
"""
from .binding import (  # noqa: F401
    SVG2_BF16, SVG2_F32, Svg2Error, load_library, svg2_forward, svg2_forward_gather_free,
    svg2_forward_workspace_size,
    svg2_kmeans, svg2_permute, svg2_permute_noalloc, svg2_profile_enable, svg2_profile_read, svg2_profile_read_kernels, svg2_select_topp, svg2_sparse_attn,
    svg2_sparse_attn_gather_free, svg2_attention_recall, svg2_kmeans_pp_init,
    svg2_quantize_fp8, svg2_sparse_attn_fp8, svg2_forward_fp8,
)
