"""MI355X-native low-precision (Qm.f fixed-point) forward path: thin Python binding over
the C-ABI library liblp.so declared in include/lp.h.  All arithmetic runs in the HIP
kernels; this package only marshals arguments (torch is used for device memory and streams).
"""
from .binding import (  # noqa: F401
    LP_RANGE_WORKSPACE_WORDS,
    LP_ROUND_NEAREST_AWAY,
    LP_ROUND_NEAREST_EVEN,
    LP_ROUND_STOCHASTIC,
    LP_STATIC_WORKSPACE_BYTES,
    ConvDesc,
    LpError,
    QFmt,
    exported_symbols,
    lib_path,
    load,
    lp_act,
    lp_act_stochastic,
    lp_conv_fwd,
    lp_conv_fwd_static,
    lp_conv_pack_weights,
    lp_conv_packed_bytes,
    lp_conv_plan_info,
    lp_conv_workspace_bytes,
    lp_fc_fwd,
    lp_fc_pack_weights,
    lp_fc_packed_bytes,
    lp_fc_workspace_bytes,
    lp_maxpool2x2,
    lp_quantize,
    lp_range,
    lp_range_acc,
    lp_status_string,
)
