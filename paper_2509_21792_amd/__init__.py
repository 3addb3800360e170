"""MI355X-native speculative-verify hot path of FastGRPO's generation phase (C-ABI HIP library + thin binding)."""
from .binding import (ACCEPT_GREEDY, ACCEPT_REJECT, ACCEPT_SAMPLE_MATCH, FG_BF16, FG_F16, FG_F32, FG_MAX_NODES, FgError, KVCache,  # noqa: F401
                      Model, fg_attention, fg_build_tree, fg_topk_logp, fg_lm_head_topk, fg_draft_frontier, fg_draft_step, fg_gemm, fg_kv_compact,
                      fg_knee, fg_pack_weight, fg_plan, fg_select_rows, fg_model_profile, fg_model_profile_read, fg_gemm_kernel_name, fg_spec_accept, fg_spec_accept_static, fg_draft_train_grad, fg_draft_train_pack_head, fg_draft_adamw, draft_param_shapes, fg_spec_verify, fg_probe_read,
                      fg_probe_copy, fg_probe_mfma, STATIC_SCRATCH_BYTES, lib)
