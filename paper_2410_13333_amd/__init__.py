"""MI355X-native decoder-stage forward/backward: the per-GPU compute of a hybrid-parallel training step
with a run-time layer count and micro-batch count.  Thin ctypes binding over libmls.so (include/mls.h)."""
from .binding import (  # noqa: F401
    MlsError, MlsConfig, MlsMemory, Stage, gemm, lib, lib_path, P_NAMES, T_IDS, MLS_BF16, MLS_FP32,
    Ends, MlsEndsConfig, PE_NAMES, Optim, Probe, MlsAdamW,
    plan_layers, plan_layer_cap, plan_split_groups, plan_microbatches, plan_lower_level, grouping_time_ratio, theoretic_slowdown,
)
