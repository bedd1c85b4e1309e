"""ARRoL online rollout-pruning data path for AMD MI355X (gfx950).

The product is libarrol.so (hand-written HIP, C ABI in include/arrol.h); this package is
its thin Python binding.  The library is loaded on first use and there is no fallback.
"""
from .binding import (ArrolError, KVLayout, Policy, arrol_calibrate, arrol_histogram, arrol_prune_bernoulli, arrol_probe_mfma_rate, LIB_PATH, MAX_GROUP, arrol_compact, arrol_compact_inplace, arrol_compact_static, arrol_compact_workspace_bytes,
                      arrol_logprob, arrol_logprob_workspace_bytes, arrol_score, arrol_score_grad, arrol_adamw_step, arrol_score_mlp, arrol_score_mlp_grad, arrol_select,
                      arrol_weighted_vote, arrol_grpo_advantage, arrol_grpo_objective, arrol_token_confidence, arrol_trace_confidence, error_string, kv_layout_of, lib, version)
