"""warmkv: MI355X-native KV-cache reclaim (plan, compact, remap) and weight
materialisation behind a C ABI (include/warmkv.h, libwarmkv.so)."""
from .binding import (KV_E_ALIGN, KV_E_BADPLAN, KV_E_HIP, KV_E_NOSPACE, KV_E_NULL, KV_E_OVERLAP, KV_E_RANGE,
                      KV_E_TOOBIG, KV_OK, StaleLibraryError, WarmKVError, warmkv_build_id, kv_compact, kv_compact_launch, kv_plan_bind,
                      kv_grow, kv_plan_fetch, kv_plan_reclaim, kv_plan_workspace_bytes, kv_remap_tables,
                      kv_reserve_blocks, kv_switch, kv_compact_moves, kv_movers_in_front, weights_materialize_front,
                      kv_vmm_kv_base, kv_vmm_pool_create, kv_vmm_pool_destroy,
                      kv_vmm_reclaim, kv_vmm_restore, kv_vmm_slot_base, pool_desc, warmkv_version, weights_materialize,
                      weights_materialize_pipelined, weights_materialize_schedule, make_model,
                      ws_place_replicas, ws_predict_load, ws_replica_scores)

__all__ = ["KV_OK", "KV_E_NULL", "KV_E_RANGE", "KV_E_ALIGN", "KV_E_TOOBIG", "KV_E_OVERLAP", "KV_E_HIP",
           "KV_E_NOSPACE", "KV_E_BADPLAN", "WarmKVError", "pool_desc", "kv_plan_workspace_bytes",
           "kv_plan_bind", "kv_plan_reclaim", "kv_compact", "kv_compact_launch", "kv_remap_tables",
           "kv_plan_fetch", "weights_materialize", "weights_materialize_schedule", "weights_materialize_pipelined",
           "kv_switch", "kv_compact_moves", "kv_movers_in_front", "weights_materialize_front", "kv_reserve_blocks", "kv_grow", "kv_vmm_pool_create", "kv_vmm_kv_base", "kv_vmm_slot_base",
           "kv_vmm_reclaim", "kv_vmm_restore", "kv_vmm_pool_destroy", "make_model", "ws_predict_load",
           "ws_replica_scores", "ws_place_replicas", "warmkv_version", "warmkv_build_id", "StaleLibraryError"]
