"""MI355X-native sparsely activated expert FFN layer with weight-only int4/int8 experts.

The work is done by the HIP library behind ``include/moe_wq.h``; ``binding`` marshals torch
device pointers into its C entry points (loaded on first use, and failing loudly if the
library has not been built).  ``workloads`` holds the seeded synthetic input generators.
"""

from . import binding, layer, workloads  # noqa: E402,F401
from .layer import MoEExpertLayer  # noqa: E402,F401
from .binding import (MoeError, moe_combine, moe_gate_topk, moe_grouped_ffn_wq,  # noqa: E402,F401
                      moe_grouped_ffn_wq_workspace_bytes, moe_permute, moe_permute_workspace_bytes,
                      moe_quantize_experts)
