"""CPU oracle (test infrastructure only; see arrol_oracle.py)."""
from .arrol_oracle import (bf16_bits_to_f64, score, quantise, select_group, select,
                           compact, log_softmax_rows, logprob, weighted_vote,
                           FIXED_POINT_BITS, bin_index, histogram, posterior_lut, bin_weights,
                           survival_lut, calibrate, prune_bernoulli, compact_inplace, score_mlp,
                           score_ce, score_ce_grad, adamw_step,
                           token_confidence, trace_confidence, grpo_advantage, grpo_objective, score_mlp_ce_grad)
