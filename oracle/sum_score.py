"""Oracle: the probability of a collapsed draft summed over all of its alignments (Eq. 5), as an alternative
value of a candidate to the best single alignment of Eq. 6.

Test infrastructure only (see the package docstring).

Eq. 5 sums P(A|X) over every raw sequence A of T tokens, drawn from the whole vocabulary plus the blank, that
the collapse rule turns into Y; with Eq. 6 each P(A|X) is a product over the slots.  The sum is computed by
the forward recursion of the connectionist-temporal-classification paper that Sec. 3.2 cites, over the
extended sequence blank, y1, blank, y2, ..., blank, in log space.
"""
import numpy as np


def ctc_sequence_logprob(logp, y, blank):
    """log P(Y|X): logp [T, V+1] float log-probabilities of every token (and the blank) per slot, y a tuple
    of tokens without blanks.  -inf when Y cannot be reached in T slots."""
    logp = np.asarray(logp, dtype=np.float64)
    T = logp.shape[0]
    z = [blank]
    for tok in y:
        z += [int(tok), blank]
    S = len(z)
    alpha = np.full(S, -np.inf)
    alpha[0] = logp[0, z[0]]
    if S > 1:
        alpha[1] = logp[0, z[1]]
    for t in range(1, T):
        new = np.full(S, -np.inf)
        for s in range(S):
            a = alpha[s]                       # stay on the same symbol
            if s >= 1:
                a = np.logaddexp(a, alpha[s - 1])  # advance by one
            if s >= 2 and z[s] != blank and z[s] != z[s - 2]:
                a = np.logaddexp(a, alpha[s - 2])  # skip the blank between two different tokens
            new[s] = a + logp[t, z[s]]
        alpha = new
    total = alpha[S - 1]
    if S > 1:
        total = np.logaddexp(total, alpha[S - 2])
    return float(total)


def sum_scores(logits, lse, cand_tokens, cand_len, n_cand, blank):
    """Eq. 5 value of every candidate of one sequence.  logits [T, V+1] and lse [T] (any float dtype, used as
    they are: log p = logit - lse); cand_tokens [beam, T], cand_len [beam].  Returns float64 [beam], -inf
    beyond n_cand."""
    logits = np.asarray(logits, dtype=np.float64)
    lse = np.asarray(lse, dtype=np.float64)
    logp = logits - lse[:, None]
    out = np.full(cand_tokens.shape[0], -np.inf)
    for i in range(int(n_cand)):
        y = tuple(int(v) for v in cand_tokens[i, : int(cand_len[i])])
        out[i] = ctc_sequence_logprob(logp, y, blank)
    return out


def ranks_desc(values, n):
    """Rank of each of the first n values in the order (value descending, index ascending); -1 beyond n.
    Values are compared as given (the caller passes the precision the decision is taken in)."""
    values = np.asarray(values)
    rank = np.full(values.shape[0], -1, dtype=np.int32)
    order = sorted(range(int(n)), key=lambda i: (-float(values[i]), i))
    for r, i in enumerate(order):
        rank[i] = r
    return rank
