"""MI355X-native static-tree Medusa verification (libmedusa_hip + a thin ctypes binding)."""
from .binding import (EXPORTED, LIB_PATH, MDZ_BF16, MDZ_FP32, MDZ_FP16, MDZ_KV_PLAIN, MDZ_KV_FP8E4M3, KV_QUANT, MDZ_TREE_15, MDZ_TREE_64, MDZ_TREE_1, MDZ_TREE_64_K5, DTYPES, TREES, KvDesc,
                      LayerWeights, MedusaError, ModelDesc, Weights, accept_longest_prefix, kv_compact, lib,
                      medusa_heads, medusa_kv_bytes, medusa_kv_init, medusa_test_force_unfused_rope, MDZ_STATUS_SEQ_RANGE, medusa_kv_read, medusa_kv_write, medusa_pack_tile_rows,
                      medusa_pack_weight, medusa_pack_weight_bf16_as_f16, medusa_packed_bytes, medusa_profile_begin, medusa_profile_end, medusa_stream_copy, medusa_stream_read, medusa_tree_info, medusa_tree_tables,
                      medusa_workspace_bytes, medusa_gemm_plan, medusa_gemm_slot_count, tree_verify_layer, tree_verify_layer_static, tree_verify_layer_static_scratch_bytes, tree_verify_step)
from .runtime import ChainedDecoder, DeviceKV, DeviceModel, StepBuffers, run_step
