"""MI355X-native AsyncMesh stage update: fused optimizer step + look-ahead + asynchronous sparse
averaging with EMA delay correction, as a C-ABI HIP library with a thin binding.

The binding (and with it the built library) is loaded on first use of one of its names, so that
`paper_2601_22442_amd.build` can be imported in a tree where nothing is built yet.  There is no
fallback: without libasyncmesh.so every name of the binding raises ImportError."""
from .schedules import active_mask, ema_lambda, learning_rate  # noqa: F401

_BINDING_NAMES = (
    "BF16", "CORR_EAGER", "CORR_EMA", "CORR_NONE", "F32", "MAX_REPLICAS", "MSG_BF16", "MSG_E4M3", "MSG_F32",
    "OPT_ADAMW", "OPT_NADAMW", "OPT_SGD", "SUBSET_BERNOULLI", "SUBSET_STRATIFIED", "D_PER_REPLICA", "D_INTERLEAVED",
    "d_layout_info",
    "AsyncMeshError", "Config", "Snapshot", "Stage", "init_state", "lookahead", "make_config", "version",
    "workspace_bytes",
)


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")


def __dir__():
    return sorted(list(globals()) + list(_BINDING_NAMES))
