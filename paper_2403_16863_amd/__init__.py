"""MI355X-native fused attention forward (C-ABI library + thin binding)."""
from .binding import (ATTN_BF16, ATTN_F16, AttnError, attn_codeobj_load, attn_codeobj_unload,  # noqa: F401
                      attn_default_variant, attn_deploy_clear, attn_deploy_codeobj, attn_deploy_variant,
                      attn_deployed, attn_fwd, attn_fwd_codeobj, attn_time_codeobj,
                      attn_fwd_variant, attn_knob_name, attn_knob_size, attn_mfma_ceiling, attn_mix_ceiling,
                      attn_num_knobs, attn_num_variants, attn_schedule_grid, attn_schedule_item, attn_valu_ceiling,
                      attn_time_variant, attn_variant_coords, attn_variant_desc,
                      attn_variant_from_coords, attn_variant_supported)
