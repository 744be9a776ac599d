"""MI355X-native MoE expert layer (one FFN-group GPU's share): thin binding over the
hand-written HIP library libmoe_mi355x.so.  Nothing here computes anything; the binding
raises if the library has not been built."""
from .binding import (  # noqa: F401
    MOE_BF16, MOE_F32, GATE_SIGMOID_RENORM, GATE_SOFTMAX, GATE_SOFTMAX_RENORM,
    MoeError, lib_path, load_library, moe_combine, moe_dispatch, moe_expert_bwd,
    moe_expert_fwd, moe_route, moe_workspace_bytes,
)
