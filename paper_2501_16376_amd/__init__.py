"""SwiftPrune per-layer pruning path for AMD MI355X (gfx950).

The work is done by hand-written HIP kernels behind a C ABI
(``include/swiftprune.h``, built into ``libswiftprune.so``); :mod:`.binding`
marshals torch device tensors into those calls and :mod:`.synth` generates
seeded synthetic layers.  There is no CPU fallback: calling an entry point
without the built library or without a GPU raises.
"""
__version__ = "0.1.0"

_BINDING_NAMES = (
    "swiftprune_layer_stats", "swiftprune_score_select", "swiftprune_nm_select", "swiftprune_apply",
    "swiftprune_layer_stats_static", "swiftprune_score_select_group", "swiftprune_nm_select_group",
    "swiftprune_calibrate_la_device", "swiftprune_la_workspace_bytes", "swiftprune_score_select_la", "prune_group",
    "swiftprune_channel_factor", "swiftprune_layer_stats_from_partials", "swiftprune_ewma_trace", "swiftprune_count_pruned", "swiftprune_calibrate_la", "swiftprune_topk_select", "swiftprune_compact_nm", "swiftprune_expand_nm",
    "swiftprune_nm_meta_words", "swiftprune_la_for_sparsity", "swiftprune_stats_workspace_bytes", "swiftprune_strerror",
    "swiftprune_version", "SwiftPruneError", "load_library", "prune_layer", "LayerBuffers",
    "SP_SEQUENTIAL_ORDER", "SP_APPLY_INPLACE", "SP_F32", "SP_BF16", "SP_F16",
)


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
