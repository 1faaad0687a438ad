"""CPU pins of the Eq. 5 (sum over alignments) oracle: hand cases, the definition by brute force over every
raw sequence, total probability, torch's CTC loss, and the bound by the best alignment."""
import itertools
import math

import numpy as np
import pytest
import torch

import oracle


def _logp(seed, T, C):
    rng = np.random.default_rng(seed)
    z = rng.standard_normal((T, C)) * 2.0
    return z - np.log(np.exp(z).sum(-1, keepdims=True))


def test_hand_cases():
    lp = _logp(0, 2, 3)  # tokens 0, 1; blank 2
    p = np.exp(lp)
    # one slot would give p(y); two slots, Y = (0): "0 0", "0 _", "_ 0"
    assert math.isclose(oracle.ctc_sequence_logprob(lp[:1], (0,), 2), lp[0, 0], rel_tol=1e-14)
    want = p[0, 0] * p[1, 0] + p[0, 0] * p[1, 2] + p[0, 2] * p[1, 0]
    assert math.isclose(math.exp(oracle.ctc_sequence_logprob(lp, (0,), 2)), want, rel_tol=1e-13)
    # Y = (0, 1): only "0 1";  Y = (0, 0) needs a blank between: impossible in two slots;  Y = (): "_ _"
    assert math.isclose(oracle.ctc_sequence_logprob(lp, (0, 1), 2), lp[0, 0] + lp[1, 1], rel_tol=1e-14)
    assert oracle.ctc_sequence_logprob(lp, (0, 0), 2) == -np.inf
    assert math.isclose(oracle.ctc_sequence_logprob(lp, (), 2), lp[0, 2] + lp[1, 2], rel_tol=1e-14)
    # three slots, Y = (0, 0): exactly "0 _ 0"
    lp3 = _logp(1, 3, 3)
    assert math.isclose(oracle.ctc_sequence_logprob(lp3, (0, 0), 2), lp3[0, 0] + lp3[1, 2] + lp3[2, 0], rel_tol=1e-14)


@pytest.mark.parametrize("T,V,blank", [(4, 3, 3), (5, 3, 0), (6, 2, 1)])
def test_equals_the_sum_over_every_raw_sequence(T, V, blank):
    """Eq. 5 literally: enumerate all (V+1)^T raw sequences, collapse each, add up their Eq. 6 probabilities."""
    lp = _logp(T * 10 + V, T, V + 1)
    total = {}
    for a in itertools.product(range(V + 1), repeat=T):
        y = oracle.ctc_collapse(list(a), blank)
        total[y] = total.get(y, 0.0) + math.exp(sum(lp[t, a[t]] for t in range(T)))
    assert math.isclose(sum(total.values()), 1.0, rel_tol=1e-12)
    for y, p in total.items():
        assert math.isclose(math.exp(oracle.ctc_sequence_logprob(lp, y, blank)), p, rel_tol=1e-11), y
    # a sequence no raw sequence collapses to: longer than T
    assert oracle.ctc_sequence_logprob(lp, tuple([1 if blank != 1 else 2] * (T + 1)), blank) == -np.inf


def test_against_torch_ctc_loss():
    T, C, blank = 8, 11, 10
    lp = _logp(7, T, C)
    rng = np.random.default_rng(8)
    for L in range(1, 6):
        y = tuple(int(v) for v in rng.integers(0, C - 1, size=L))
        loss = torch.nn.functional.ctc_loss(torch.from_numpy(lp)[:, None, :], torch.tensor([y]), torch.tensor([T]),
                                            torch.tensor([L]), blank=blank, reduction="sum", zero_infinity=False)
        got = oracle.ctc_sequence_logprob(lp, y, blank)
        if math.isinf(float(loss)):
            assert got == -np.inf
        else:
            assert math.isclose(got, -float(loss), rel_tol=1e-10, abs_tol=1e-10), (y, got, float(loss))


def test_sum_is_at_least_the_best_alignment_and_ranks():
    T, k, blank = 4, 3, 20
    rng = np.random.default_rng(3)
    logits = rng.standard_normal((T, 21)).astype(np.float32) * 3
    lse = np.log(np.exp(logits.astype(np.float64)).sum(-1))
    logp = logits - lse[:, None]
    ids = np.argsort(-logits, axis=-1)[:, :k]
    ids[1, 2] = blank
    top_lp = np.take_along_axis(logp, ids, axis=-1).astype(np.float32)
    drafts = oracle.collapse_candidates(ids, top_lp, blank, beam=16)
    toks = np.full((16, T), -1, dtype=np.int32)
    lens = np.zeros(16, dtype=np.int32)
    for i, (y, s, _) in enumerate(drafts):
        toks[i, :len(y)], lens[i] = y, len(y)
    sums = oracle.sum_scores(logits, lse, toks, lens, len(drafts), blank)
    for i, (y, s, _) in enumerate(drafts):
        assert sums[i] >= float(s) - 1e-5  # the best alignment is one term of the sum
    assert np.all(np.isneginf(sums[len(drafts):]))
    r = oracle.ranks_desc(sums, len(drafts))
    assert sorted(r[:len(drafts)]) == list(range(len(drafts))) and np.all(r[len(drafts):] == -1)
    assert all(sums[i] >= sums[j] for i in range(len(drafts)) for j in range(len(drafts)) if r[i] < r[j])
    # ties go to the smaller index
    assert list(oracle.ranks_desc(np.array([1.0, 2.0, 2.0, 0.5]), 4)) == [2, 0, 1, 3]
