"""CPU oracle for the CTC-drafted speculative decoding step.  TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 numpy implementation of what one draft+verify step computes
(Sec. 3.1 "Model Structure" and Sec. 3.3 "Inference" of the paper; the CTC collapse of
Sec. 2.2), written from the definitions so that it can be checked against the paper by
eye.  It shares no code with the HIP path and must never be imported by it: only the
tests, the smoke check and the benchmark's CPU-baseline leg may use this package.

Every function is pinned by the CPU tests to something other than itself (hand cases of
the collapse rule, brute-force enumeration, closed forms, textbook special cases,
structural invariants); nothing here is "parity unpinned".
"""
from .draft import lm_head_logits, log_softmax, topk_per_slot, draft_topk  # noqa: F401
from .collapse import (  # noqa: F401
    ctc_collapse,
    alignment_ranks,
    alignment_scores_f32,
    collapse_candidates,
)
from .tree import build_prefix_tree, ancestor_mask, pack_mask_u64, collapse_tree, raw_tree  # noqa: F401
from .attention import tree_attention  # noqa: F401
from .accept import accept_longest, verifier_argmax  # noqa: F401
from .verify import verifier_head_argmax, argmax_rows, kv_commit  # noqa: F401
from .draft_layer import draft_layer, draft_layer_qkv, draft_layer_attend, rms_norm, rope, silu  # noqa: F401
from .sum_score import ctc_sequence_logprob, sum_scores, ranks_desc  # noqa: F401
from .ctc_loss import ctc_alpha_beta, ctc_loss_and_grad  # noqa: F401
from .sampling import (  # noqa: F401
    target_probs,
    sample_token,
    sample_nodes,
    accept_sampled,
    sec2_rule_distribution,
    sample_and_match_distribution,
)
