"""MI355X-native FAAR layer-step library: hand-written HIP kernels behind a C ABI (libfaar.so)
plus a ctypes binding.  Importing the package does not load the library; the first call does,
and raises if it has not been built."""
from .binding import (FaarError, faar_adam, faar_harden_pack, faar_hardened_loss, faar_init_v,  # noqa: F401
                      faar_layer_prepare, faar_stochastic_v,
                      faar_layer_step, faar_padded_tokens, faar_dw_token_major, faar_quant_rtn, faar_softquant_fwd_bwd,
                      faar_softquant_fwd_bwd_static, faar_gemm_plan, tensor_batch, faar_quant_rtn_batch,
                      faar_init_v_batch, faar_harden_pack_batch, faar_linear_forward, faar_rmsnorm_fwd, faar_rmsnorm_bwd,
                      faar_silu_mul_fwd, faar_silu_mul_bwd, faar_block_output_loss, faar_residual_add, faar_rope, block_description, faar_block_workspace, faar_block_joint_step, faar_attention_fwd, faar_attention_bwd,
                      faar_stage2_losses, faar_workspace_bytes, layer_step_workspace, lib)
