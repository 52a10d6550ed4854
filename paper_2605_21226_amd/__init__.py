"""MI355X-native OCTOPUS key codec and fused decode attention (C-ABI library + thin binding)."""
from .binding import (Codebooks, OctopusError, Plan, load, octopus_attn_decode, octopus_attn_decode_workspace,  # noqa: F401
                      octopus_build_codebooks, octopus_build_codebooks_pair, octopus_cache_bytes, octopus_encode,
                      octopus_profile_events, octopus_qjl_bytes, octopus_encode_qjl, octopus_attn_decode_qjl, octopus_encode_rounding, octopus_vq_row_bytes, octopus_vq_bytes,
                      octopus_encode_values, octopus_attn_decode_vq, octopus_attn_decode_hybrid,
                      octopus_attn_decode_static, octopus_paged_pool_bytes, octopus_encode_paged,
                      octopus_attn_decode_paged, octopus_attn_decode_paged_hybrid, octopus_encode_values_paged,
                      octopus_attn_decode_paged_vq, octopus_encode_qjl_paged, octopus_attn_decode_paged_qjl,
                      octopus_vq_on_matrix_cores)
