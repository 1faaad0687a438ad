"""Oracle: the CTC training objective of Sec. 3.2 - the negative log of Eq. 5 for a label sequence, and its
gradient with respect to the logits - by the forward-backward recursions of the CTC paper the section cites.

Test infrastructure only (see the package docstring).

Everything is float64 and in log space, one sequence at a time.  alpha_t(s): log-probability of all prefixes
of alignments that are in state s of the extended sequence (blank, y1, blank, ..., blank) after frame t;
beta_t(s): log-probability of all suffixes that start in state s at frame t (frame t's emission included in
both).  Eq. 5: P(Y|X) = alpha_T(S-1) + alpha_T(S-2) (in probabilities).
"""
import numpy as np


def _extended(y, blank):
    z = [blank]
    for tok in y:
        z += [int(tok), blank]
    return z


def ctc_alpha_beta(logp, y, blank):
    """logp [T, V+1] log-probabilities, y label tokens.  Returns (alpha [T, S], beta [T, S], log P)."""
    logp = np.asarray(logp, dtype=np.float64)
    T = logp.shape[0]
    z = _extended(y, blank)
    S = len(z)
    skip = [s >= 2 and z[s] != blank and z[s] != z[s - 2] for s in range(S)]
    alpha = np.full((T, S), -np.inf)
    alpha[0, 0] = logp[0, z[0]]
    if S > 1:
        alpha[0, 1] = logp[0, z[1]]
    for t in range(1, T):
        for s in range(S):
            a = alpha[t - 1, s]
            if s >= 1:
                a = np.logaddexp(a, alpha[t - 1, s - 1])
            if skip[s]:
                a = np.logaddexp(a, alpha[t - 1, s - 2])
            alpha[t, s] = a + logp[t, z[s]]
    beta = np.full((T, S), -np.inf)
    beta[T - 1, S - 1] = logp[T - 1, z[S - 1]]
    if S > 1:
        beta[T - 1, S - 2] = logp[T - 1, z[S - 2]]
    for t in range(T - 2, -1, -1):
        for s in range(S):
            b = beta[t + 1, s]
            if s + 1 < S:
                b = np.logaddexp(b, beta[t + 1, s + 1])
            if s + 2 < S and skip[s + 2]:
                b = np.logaddexp(b, beta[t + 1, s + 2])
            beta[t, s] = b + logp[t, z[s]]
    total = alpha[T - 1, S - 1]
    if S > 1:
        total = np.logaddexp(total, alpha[T - 1, S - 2])
    return alpha, beta, float(total)


def ctc_loss_and_grad(logits, y, blank):
    """Loss -log P(Y|X) of one sequence and its gradient with respect to the logits [T, V+1] (the
    log-softmax is part of the differentiated function).  d loss / d logit[t, v] = softmax[t, v] -
    (sum over the states s with symbol v of alpha_t(s) beta_t(s) / p_t(v)) / P.  When Y cannot be reached
    (P = 0) the loss is +inf and the gradient is returned as zeros."""
    logits = np.asarray(logits, dtype=np.float64)
    m = logits.max(axis=-1, keepdims=True)
    lse = m + np.log(np.exp(logits - m).sum(axis=-1, keepdims=True))
    logp = logits - lse
    alpha, beta, total = ctc_alpha_beta(logp, y, blank)
    if np.isneginf(total):
        return np.inf, np.zeros_like(logits)
    z = _extended(y, blank)
    grad = np.exp(logp)
    for t in range(logits.shape[0]):
        for s, v in enumerate(z):
            ab = alpha[t, s] + beta[t, s]
            if not np.isneginf(ab):
                grad[t, v] -= np.exp(ab - logp[t, v] - total)
    return -total, grad
