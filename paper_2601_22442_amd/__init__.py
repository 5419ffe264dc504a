"""MI355X-native AsyncMesh stage update: fused optimizer step + look-ahead + asynchronous sparse
averaging with EMA delay correction, as a C-ABI HIP library with a thin binding."""
from .binding import (  # noqa: F401
    BF16, CORR_EAGER, CORR_EMA, CORR_NONE, F32, MAX_REPLICAS, MSG_BF16, MSG_E4M3, MSG_F32, OPT_ADAMW, OPT_NADAMW, OPT_SGD,
    SUBSET_BERNOULLI, SUBSET_STRATIFIED,
    AsyncMeshError, Config, Snapshot, Stage, init_state, lookahead, make_config, version, workspace_bytes,
)
from .schedules import active_mask, ema_lambda, learning_rate  # noqa: F401,E402
