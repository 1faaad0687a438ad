"""Oracle, CTC transform: enumerate slot combinations, score them, collapse, dedupe, keep the best.

Test infrastructure only (see the package docstring).
"""
import numpy as np


def ctc_collapse(a, blank):
    """The collapse map beta^-1 of Sec. 2.2: first merge every run of adjacent equal symbols
    (runs of blanks included) into one symbol, then delete the blanks.  Order matters:
    (a, blank, a) -> (a, a) while (a, a, blank, b) -> (a, b).  Returns a tuple of ints."""
    merged = []
    for s in a:
        s = int(s)
        if not merged or s != merged[-1]:
            merged.append(s)
    return tuple(s for s in merged if s != blank)


def alignment_ranks(T, k):
    """All rank tuples r in {0..k-1}^T as an int64 array [k^T, T], row idx holding the tuple with
    idx = sum_t r_t * k^(T-1-t) (slot 0 most significant).  Every raw candidate has the same
    length T (Sec. 3.1)."""
    idx = np.arange(k ** T, dtype=np.int64)
    r = np.empty((k ** T, T), dtype=np.int64)
    for t in range(T):
        r[:, t] = (idx // (k ** (T - 1 - t))) % k
    return r


def alignment_scores_f32(topk_logp, ranks):
    """log of Eq. 6, P(A|X) = prod_t p(a_t|X): the sum over slots of the chosen tokens'
    log-probabilities.  The sum is taken in float32, left to right, (((l_0 + l_1) + l_2) + ...),
    which is the precision and order in which the step ranks candidates; returns float32 [k^T]."""
    lp = np.asarray(topk_logp, dtype=np.float32)
    T = lp.shape[0]
    s = lp[0, ranks[:, 0]].astype(np.float32)
    for t in range(1, T):
        s = (s + lp[t, ranks[:, t]]).astype(np.float32)
    return s


def collapse_candidates(topk_id, topk_logp, blank, beam):
    """Candidate drafts of one sequence (Sec. 3.3: tokens of every place are combined, the most
    valuable combinations are kept and passed through the CTC transform).

    topk_id [T,k] ints, topk_logp [T,k] float32 (descending per slot).  Every one of the k^T slot
    combinations is a raw candidate; its value is its Eq. 6 log-probability.  Raw candidates are
    collapsed by beta^-1; raw candidates with the same collapsed sequence are one draft whose score is
    that of its best raw candidate and whose representative is, among the best-scoring ones, the raw
    candidate of smallest idx.  The empty draft (all blanks) is dropped.  Drafts are ordered by
    (score descending, representative idx ascending) and the first `beam` are kept.

    Returns a list of (tokens tuple, score np.float32, representative idx)."""
    ids = np.asarray(topk_id)
    T, k = ids.shape
    ranks = alignment_ranks(T, k)
    raw = ids[np.arange(T)[None, :], ranks]          # [k^T, T] raw candidate sequences
    score = alignment_scores_f32(topk_logp, ranks)   # [k^T]
    best = {}
    for idx in range(raw.shape[0]):                  # idx ascending: a strict '>' keeps the smallest idx
        y = ctc_collapse(raw[idx], blank)
        if not y:
            continue
        cur = best.get(y)
        if cur is None or score[idx] > cur[0]:
            best[y] = (score[idx], idx)
    drafts = sorted(best.items(), key=lambda kv: (-float(kv[1][0]), kv[1][1]))
    return [(y, s, idx) for y, (s, idx) in drafts[:beam]]
