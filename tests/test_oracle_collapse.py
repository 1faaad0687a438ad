"""Pins for the oracle's CTC transform (collapse, scoring, dedupe, selection).  CPU only."""
import heapq
import itertools
import math
import os

import numpy as np
import pytest

import oracle
import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "collapse_cases.txt")


def _golden_cases():
    cases = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            raw, out = line.split("->")
            cases.append((raw.split(), [] if out.strip() == "." else out.split()))
    return cases


@pytest.mark.parametrize("raw,expected", _golden_cases())
def test_collapse_hand_cases(raw, expected):
    symbols = sorted(set(raw) - {"_"})
    code = {s: i + 1 for i, s in enumerate(symbols)}
    blank = 0
    a = [blank if s == "_" else code[s] for s in raw]
    assert list(oracle.ctc_collapse(a, blank)) == [code[s] for s in expected]


def test_collapse_equals_groupby_form():
    # textbook statement of the same map: keys of itertools.groupby, blanks filtered out
    rng = np.random.Generator(np.random.PCG64(0))
    for _ in range(300):
        a = rng.integers(0, 4, size=rng.integers(1, 10)).tolist()
        ref = tuple(key for key, _ in itertools.groupby(a) if key != 3)
        assert oracle.ctc_collapse(a, 3) == ref


def test_alignment_ranks_is_counting_in_base_k():
    r = oracle.alignment_ranks(3, 4)
    assert r.shape == (64, 3)
    assert [tuple(x) for x in r.tolist()] == list(itertools.product(range(4), repeat=3))


def _f32_sum_left_to_right(vals):
    s = np.float32(vals[0])
    for v in vals[1:]:
        s = np.float32(s + np.float32(v))
    return s


def _brute_force(ids, logp, blank, beam):
    """Dictionary over every slot combination, written with itertools only."""
    T, k = ids.shape
    best = {}
    for idx, r in enumerate(itertools.product(range(k), repeat=T)):
        raw = [int(ids[t, r[t]]) for t in range(T)]
        s = float(_f32_sum_left_to_right([logp[t, r[t]] for t in range(T)]))
        y = tuple(key for key, _ in itertools.groupby(raw) if key != blank)
        if not y:
            continue
        if y not in best or s > best[y][0]:
            best[y] = (s, idx)
    order = sorted(best, key=lambda y: (-best[y][0], best[y][1]))[:beam]
    return [(y, best[y][0], best[y][1]) for y in order]


def _sorted_walk(ids, logp, blank, beam):
    """Second statement of the selection: walk raw candidates in (score desc, idx asc) order and keep
    first occurrences of non-empty collapsed sequences until `beam` are held."""
    T, k = ids.shape
    ranks = oracle.alignment_ranks(T, k)
    score = oracle.alignment_scores_f32(logp, ranks)
    order = np.lexsort((np.arange(len(score)), -score.astype(np.float64)))
    seen, out = set(), []
    for idx in order:
        y = oracle.ctc_collapse(ids[np.arange(T), ranks[idx]], blank)
        if y and y not in seen:
            seen.add(y)
            out.append((y, float(score[idx]), int(idx)))
            if len(out) == beam:
                break
    return out


@pytest.mark.parametrize("seed", range(12))
def test_candidates_match_brute_force_and_sorted_walk(seed):
    rng = np.random.Generator(np.random.PCG64(100 + seed))
    T, k = int(rng.integers(1, 6)), int(rng.integers(1, 4))
    blank = 9
    ids, logp = workloads.make_topk_case(seed, 1, T, k, blank, vocab=5, p_blank=0.6,
                                         quantum=0.5 if seed % 2 else 0.0)
    for beam in (1, 3, 1000):
        got = [(y, float(s), i) for y, s, i in oracle.collapse_candidates(ids[0], logp[0], blank, beam)]
        assert got == _brute_force(ids[0], logp[0], blank, beam)
        assert got == _sorted_walk(ids[0], logp[0], blank, beam)


def test_candidates_sorted_walk_at_7b_shape():
    # 4^8 = 65536 raw candidates: the dictionary route and the sorted-walk route agree
    ids, logp = workloads.make_topk_case(7, 1, 8, 4, 32000, vocab=40, p_blank=0.7)
    got = [(y, float(s), i) for y, s, i in oracle.collapse_candidates(ids[0], logp[0], 32000, 128)]
    assert got == _sorted_walk(ids[0], logp[0], 32000, 128)
    assert len(got) == 128


def test_total_probability_mass_closed_form():
    # Eq. 6 makes the slots independent, so the mass of all raw candidates factorises
    ids, logp = workloads.make_topk_case(3, 1, 5, 3, 9)
    ranks = oracle.alignment_ranks(5, 3)
    s = oracle.alignment_scores_f32(logp[0], ranks).astype(np.float64)
    closed = np.prod(np.exp(logp[0].astype(np.float64)).sum(axis=1))
    assert np.exp(s).sum() == pytest.approx(closed, rel=1e-5)
    # and each score is the plain sum of its slots' terms
    for idx in (0, 17, 100, 242):
        r = ranks[idx]
        assert float(s[idx]) == pytest.approx(sum(float(logp[0, t, r[t]]) for t in range(5)), abs=1e-5)


def test_scores_are_float32_left_to_right():
    # -1, -2^-24, -2^-24: left to right each tiny term is rounded away (sum -1); right to left the two
    # tiny terms first add up to -2^-23, which survives (sum -1 - 2^-23).  The order is observable.
    tiny = np.float32(-2.0 ** -24)
    lp = np.array([[-1.0, -3.0], [tiny, -2.0], [tiny, -4.0]], dtype=np.float32)
    ranks = oracle.alignment_ranks(3, 2)
    s = oracle.alignment_scores_f32(lp, ranks)
    assert s.dtype == np.float32
    assert s[0] == np.float32(-1.0)
    assert np.float32(lp[0, 0] + np.float32(lp[1, 0] + lp[2, 0])) == np.float32(-1.0 - 2.0 ** -23)
    for idx in range(8):
        assert s[idx] == _f32_sum_left_to_right([lp[t, ranks[idx, t]] for t in range(3)])


def test_k1_is_ctc_best_path_decoding():
    # with one token per slot the only draft is the greedy CTC decode of the per-slot argmax
    rng = np.random.Generator(np.random.PCG64(5))
    for _ in range(50):
        T = int(rng.integers(1, 9))
        ids = rng.integers(0, 4, size=(T, 1))
        logp = -rng.random((T, 1)).astype(np.float32)
        ref = tuple(key for key, _ in itertools.groupby(ids[:, 0].tolist()) if key != 3)
        got = oracle.collapse_candidates(ids, logp, 3, 8)
        if ref:
            assert len(got) == 1 and got[0][0] == ref and got[0][2] == 0
            assert got[0][1] == _f32_sum_left_to_right(logp[:, 0])
        else:
            assert got == []


def test_without_blank_or_repeats_is_cartesian_top_n():
    # no blank in any list and disjoint token sets per slot: nothing collapses, so the drafts are the
    # `beam` most probable tuples of the Cartesian product (Medusa-style), each of full length T.
    T, k, beam = 5, 3, 40
    rng = np.random.Generator(np.random.PCG64(6))
    ids = (np.arange(T)[:, None] * 10 + np.arange(k)[None, :]).astype(np.int32)
    logp = -np.sort(rng.exponential(1.0, size=(T, k)), axis=1).astype(np.float32)
    got = oracle.collapse_candidates(ids, logp, 999, beam)
    assert all(len(y) == T for y, _, _ in got) and len(got) == beam
    # independent route: best-first search over rank tuples with a heap (float64 scores)
    lp = logp.astype(np.float64)
    start = (0,) * T
    heap, seen, out = [(-lp[np.arange(T), start].sum(), start)], {start}, []
    while heap and len(out) < beam:
        neg, r = heapq.heappop(heap)
        out.append((r, -neg))
        for t in range(T):
            if r[t] + 1 < k:
                n = r[:t] + (r[t] + 1,) + r[t + 1:]
                if n not in seen:
                    seen.add(n)
                    heapq.heappush(heap, (-lp[np.arange(T), n].sum(), n))
    for (y, s, idx), (r, s64) in zip(got, out):
        assert float(s) == pytest.approx(s64, abs=1e-5)
    assert {y for y, _, _ in got} == {tuple(int(ids[t, r[t]]) for t in range(T)) for r, _ in out}


def test_single_slot_gives_non_blank_tokens_in_order():
    ids = np.array([[7, 3, 5, 1]])
    logp = np.array([[-0.1, -0.5, -1.0, -2.0]], dtype=np.float32)
    got = oracle.collapse_candidates(ids, logp, 3, 10)
    assert [y for y, _, _ in got] == [(7,), (5,), (1,)]
    assert [i for _, _, i in got] == [0, 2, 3]


def test_all_blank_lists_give_no_draft():
    ids = np.full((4, 1), 50)
    logp = np.full((4, 1), -0.1, dtype=np.float32)
    assert oracle.collapse_candidates(ids, logp, 50, 8) == []


def test_tie_break_prefers_smaller_index():
    # two slots with identical lists: (a,b) and (b,a) tie exactly; (a,a)->a and (b,b)->b
    ids = np.array([[1, 2], [1, 2]])
    logp = np.array([[-0.5, -0.75], [-0.5, -0.75]], dtype=np.float32)
    got = oracle.collapse_candidates(ids, logp, 0, 10)
    assert [(y, i) for y, _, i in got] == [((1,), 0), ((1, 2), 1), ((2, 1), 2), ((2,), 3)]
    assert float(got[1][1]) == float(got[2][1]) == -1.25
