"""MI355X-native mixed-precision delta linear layer (ME-Switch serving hot path).

The package is a thin binding over libmes.so (hand-written HIP kernels for gfx950 behind a C ABI,
declared in include/mes.h).  Importing it without the built library raises ImportError.
"""
from .binding import (  # noqa: F401
    GRID_EQ1, GRID_SYM, STEP_GIVEN, STEP_MAXABS, STEP_MEANABS, DeltaLinear, MesError, PackedDelta,
    base_bytes, codes_bytes, linear_workspace_bytes, make_workspace, mes_delta_linear, mes_pack_base,
    mes_pack_delta, mes_select_salient, mes_unpack_base, mes_unpack_delta, salient_bytes, DeltaLinearMulti, KernelTimer,
    mes_copy_probe, ExpertPool, mes_delta_linear_descriptors, mes_delta_linear_multi_descriptors, StepGrad, mes_step_adamw,
    mes_delta_linear_noalloc, DeltaLinearGated,
)
