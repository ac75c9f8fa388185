"""MI355X-native (gfx950) hot path of one DySpec speculative step (arXiv 2410.11744):
``build_tree`` (Algorithm 1 + ancestor mask), ``tree_attn`` (tree-masked attention) and
``verify`` (Algorithm 3).  The work is done by hand-written HIP kernels behind the C ABI
in ``include/dyspec.h``; this package only marshals arguments."""
from .binding import (BF16, BF16_WAVE, F32, MAX_BUILD_NODES, MAX_NODES, Batch, BuiltTrees, DyspecError, PreparedCall, ReorderedTrees, Tree, VerifyOutput,
                      dfs_reorder,
                      build_tree, build_tree_threshold, init, load_library, probe_clock, probe_hbm_read, probe_mfma_bf16, status_string, tree_attn, tree_attn_call, tree_attn_layers,
                      verify, verify_call)

__all__ = ["BF16", "BF16_WAVE", "F32", "MAX_BUILD_NODES", "MAX_NODES", "Batch", "BuiltTrees", "DyspecError", "PreparedCall", "ReorderedTrees", "Tree", "VerifyOutput",
           "dfs_reorder",
           "build_tree", "build_tree_threshold", "init", "load_library", "probe_clock", "probe_hbm_read", "probe_mfma_bf16", "status_string", "tree_attn", "tree_attn_call", "tree_attn_layers",
           "verify", "verify_call"]
