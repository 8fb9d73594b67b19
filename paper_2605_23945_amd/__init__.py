"""MI355X-native decode step of one tensor-parallel shard (C-ABI library + thin binding)."""
from .binding import (  # noqa: F401
    Decoder, PatError, load_library, make_cfg, pat_cfg, pat_mem_req, pat_step_report, pat_grid_row, EXPORTS, LIB_PATH,
    pat_op_pack_weight, pat_op_pack_act, pat_op_gemm, pat_op_gemm_static, pat_op_rmsnorm_pack, pat_op_embed_stats, pat_op_pack_act_gain, pat_op_gemm_norm, pat_op_argmax, pat_op_barrier_probe, unpack_act,
    Predictor, pat_kv_move_seconds, pat_rms_length, pat_profile_plan,
)
from .synthetic import load_synthetic_weights, admit_synthetic  # noqa: F401
