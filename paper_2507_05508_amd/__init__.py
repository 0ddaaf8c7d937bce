"""MI355X-native hot path of Multilevel Monte Carlo gradient compression (arXiv 2507.05508):
HIP kernels for gfx950 behind a C ABI (include/mlmc.h), with a thin ctypes binding."""
from .binding import (  # noqa: F401
    MLMC_BF16, MLMC_BITS, MLMC_DEV_CAPACITY, MLMC_DEV_INTERNAL, MLMC_DEV_NONFINITE, MLMC_DEV_REDONE, MLMC_F32, MLMC_TILE, MLMC_TOPK,
    MLMC_ELIMIT, MLMC_FBITS, MLMC_VBITS, MLMC_RTN, mlmc_compress_rtn, MLMC_STOPK, MLMC_STATIC_SCRATCH_BYTES, mlmc_compress_bits_static, mlmc_aggregate_update, mlmc_message_bits,
    BitsMessage, MlmcError, Plan, SparseMessage, lib, mlmc_aggregate, mlmc_compress_bits, mlmc_compress_topk,
    mlmc_geometric_p, mlmc_level_norms, mlmc_plan, mlmc_profile_enable, mlmc_profile_get, mlmc_profile_reset,
)
