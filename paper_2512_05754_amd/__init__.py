"""MI355X-native dynamic block-sparse video attention (scores -> top-k -> block-sparse flash attention).

The HIP library is loaded lazily on first use of a binding function so that importing the
package (for example for its input generators) never needs the GPU.
"""

_BINDING_NAMES = (
    "block_scores",
    "block_scores_static",
    "select_topk",
    "block_sparse_attn",
    "attn_work_order",
    "merge_similarity",
    "merge_plan",
    "merge_plan_workspace_bytes",
    "merge_apply",
    "unmerge_apply",
    "attn_entropy",
    "entropy_allocate",
    "coarse_attn",
    "fuse_outputs",
    "cube_order",
    "cube_order_padded",
    "block_scores_raster",
    "block_sparse_attn_raster",
    "coarse_attn_raster",
    "cube_token_order",
    "cube_gather",
    "cube_scatter",
    "workspace_bytes",
    "lib",
    "lib_path",
    "UsvError",
    "EXPORTED_SYMBOLS",
)


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding

        return getattr(binding, name)
    raise AttributeError(name)
