"""Oracle, draft head: LM-head projection over vocabulary + blank, log-softmax, per-slot top-k.

Test infrastructure only (see the package docstring).  float64 throughout.
"""
import numpy as np


def lm_head_logits(hidden, w, bias=None):
    """Logits of every draft slot over the augmented vocabulary (Sec. 3.2, the equation
    P^ = Softmax(LmHead(F^)); the blank is one more output row, Sec. 2.2).

    hidden [..., D], w [V+1, D] (row v is token v's head vector, last row the blank),
    bias [V+1] or None (an additive logit bias).  Returns float64 [..., V+1]:
        z[..., v] = sum_d hidden[..., d] * w[v, d] + bias[v].
    """
    h = np.asarray(hidden, dtype=np.float64)
    z = h @ np.asarray(w, dtype=np.float64).T
    if bias is not None:
        z = z + np.asarray(bias, dtype=np.float64)
    return z


def log_softmax(z):
    """log of the softmax over the last axis, blank included (Sec. 3.2: P^ is a distribution over
    the augmented vocabulary for each position).  Returns (logp, lse) with logp = z - lse."""
    z = np.asarray(z, dtype=np.float64)
    m = z.max(axis=-1, keepdims=True)
    lse = m + np.log(np.exp(z - m).sum(axis=-1, keepdims=True))
    return z - lse, lse[..., 0]


def topk_per_slot(z, k):
    """Indices of the k largest entries of each row of z, in descending order of value (Sec. 3.3:
    for every position the top k tokens are taken in descending order of probability).  Equal
    values are ordered by ascending token id.  The blank competes like any other token.
    Returns int64 [..., k]."""
    z = np.asarray(z)
    # a stable sort of the negated values keeps equal values in ascending index order
    order = np.argsort(-z, axis=-1, kind="stable")
    return order[..., :k]


def draft_topk(hidden, w, bias, k):
    """Stage 1+2 of the step: logits, log-softmax, per-slot top-k.

    Returns dict with z [B,T,V+1] f64, lse [B,T] f64, topk_id [B,T,k] i64, topk_logp [B,T,k] f64."""
    z = lm_head_logits(hidden, w, bias)
    logp, lse = log_softmax(z)
    ids = topk_per_slot(z, k)
    return {
        "z": z,
        "lse": lse,
        "topk_id": ids,
        "topk_logp": np.take_along_axis(logp, ids, axis=-1),
    }
