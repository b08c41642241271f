"""MI355X-native BCQ linear layer (AlphaTuning, arXiv 2210.03858): HIP kernels behind a C ABI.

`binding` holds the thin ctypes layer over libbcq_hip.so; `synth` holds the seeded input generators.
"""
from . import synth  # noqa: F401
from .binding import (BatchPlan, BcqError, batch_plan, bcq_batch_prepare, bcq_linear_batched, bcq_prepare, abi_version, bcq_alpha_adamw_step, bcq_linear_bwd_alpha_adamw, bcq_linear_bwd_alpha, bcq_linear_bwd_alpha_grouped,  # noqa: F401
                      bcq_linear_bwd_input, bcq_linear_bwd_input_grouped, bcq_linear_fwd, bcq_linear_fwd_decode,
                      bcq_linear_fwd_grouped, bcq_linear_fwd_lut, bcq_linear_fwd_static, bcq_pack_decode, decode_layout_bytes,
                      bcq_pack, bcq_pack_transposed, bcq_quantize, bcq_quantize_alternating, bcq_quantize_grouped, bcq_unpack, load,
                      status_string, workspace_bytes, workspace_bytes_grouped)
