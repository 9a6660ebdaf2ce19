"""MI355X-native hot path of Aggressive Decoding (parallel verification and the decode
loops around it).  All compute lives in the HIP library built from csrc/; this package
only marshals arguments to its C ABI (see include/ad.h)."""
from .binding import (  # noqa: F401
    AD_BF16, AD_DRAFTER, AD_OPT_GRAPHS, AD_OPT_GRAPHS_CAPTURED, AD_OPT_SPIN_WAIT, AD_OPT_FUSE_CROSSQ, AD_OPT_OVERLAP_ENCODERS, AD_EDEVICE, AD_EINVAL, AD_ENOMEM, AD_ESTATE, AD_F32, AD_NEVER, AD_OK, AD_VERIFIER,
    AdConfig, AdError, AdStats, Context, EXPORTS, calibration_copy, calibration_mfma, LIB_PATH, config_check, host_simulate, lib, make_config,
    pack_weights, pack_weights_host, suffix_match, weights_layout, workspace_bytes,
)
