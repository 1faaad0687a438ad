"""Pins for the oracle's draft-head functions (logits, log-softmax, top-k).  CPU only."""
import math

import numpy as np
import pytest

import oracle
import workloads


def test_logits_match_exact_sums_of_products():
    # bf16 x bf16 products are exact in float64; math.fsum adds them with a single rounding, so this
    # is the exactly rounded value of the definition z = sum_d h_d * w_vd + bias_v.
    rng = np.random.Generator(np.random.PCG64(1))
    T, D, V1 = 3, 96, 7
    h = workloads.round_to_storage(rng.standard_normal((T, D), dtype=np.float32), "bf16")
    w = workloads.round_to_storage(rng.standard_normal((V1, D), dtype=np.float32), "bf16")
    bias = rng.standard_normal(V1).astype(np.float32)
    z = oracle.lm_head_logits(h, w, bias)
    assert z.shape == (T, V1) and z.dtype == np.float64
    for t in range(T):
        for v in range(V1):
            exact = math.fsum([float(h[t, d]) * float(w[v, d]) for d in range(D)] + [float(bias[v])])
            assert z[t, v] == pytest.approx(exact, rel=1e-13, abs=1e-13)


def test_logits_bias_only_and_no_bias():
    w = np.arange(12, dtype=np.float64).reshape(4, 3)
    bias = np.array([0.0, 0.0, 0.0, 1.5])
    assert np.array_equal(oracle.lm_head_logits(np.zeros((2, 3)), w, bias), np.tile(bias, (2, 1)))
    # unit vectors pick columns of w: z[t, v] = w[v, t]
    assert np.array_equal(oracle.lm_head_logits(np.eye(3), w, None), w.T)


def test_log_softmax_closed_forms():
    n = 101
    logp, lse = oracle.log_softmax(np.full((2, n), 3.25))
    assert np.allclose(logp, -math.log(n), rtol=0, atol=1e-14)
    assert np.allclose(lse, 3.25 + math.log(n), rtol=0, atol=1e-14)
    a, b = 0.3, -1.1
    logp, _ = oracle.log_softmax(np.array([a, b]))
    assert logp[0] == pytest.approx(-math.log1p(math.exp(b - a)), abs=1e-15)
    assert logp[1] == pytest.approx((b - a) - math.log1p(math.exp(b - a)), abs=1e-15)


def test_log_softmax_normalised_and_shift_invariant():
    rng = np.random.Generator(np.random.PCG64(2))
    z = rng.standard_normal((5, 333)) * 4
    logp, lse = oracle.log_softmax(z)
    assert np.allclose(np.exp(logp).sum(-1), 1.0, rtol=0, atol=1e-12)
    logp2, lse2 = oracle.log_softmax(z + 1000.0)
    assert np.allclose(logp, logp2, rtol=0, atol=1e-10)
    assert np.allclose(lse2 - lse, 1000.0, rtol=0, atol=1e-10)
    # no overflow for large logits
    logp3, _ = oracle.log_softmax(np.array([1e4, 1e4 - 1.0]))
    assert np.isfinite(logp3).all()


def _topk_by_selection(row, k):
    """k rounds of 'take the largest remaining value, smallest index among equals'."""
    taken, out = set(), []
    for _ in range(k):
        best = None
        for i, v in enumerate(row):
            if i in taken:
                continue
            if best is None or v > row[best]:
                best = i
        taken.add(best)
        out.append(best)
    return out


def test_topk_forced_ties_and_blank():
    z = np.array([[1.0, 3.0, 3.0, 2.0, 3.0], [5.0, 5.0, 5.0, 5.0, 5.0], [0.0, -1.0, 2.0, 2.0, 9.0]])
    ids = oracle.topk_per_slot(z, 3)
    assert ids.tolist() == [[1, 2, 4], [0, 1, 2], [4, 2, 3]]  # last column plays the blank: it competes


def test_topk_matches_selection_and_lexsort():
    rng = np.random.Generator(np.random.PCG64(3))
    z = np.round(rng.standard_normal((6, 50)) * 2, 1)  # coarse values: many exact ties
    k = 7
    ids = oracle.topk_per_slot(z, k)
    for t in range(z.shape[0]):
        assert ids[t].tolist() == _topk_by_selection(z[t].tolist(), k)
        full = np.lexsort((np.arange(z.shape[1]), -z[t]))
        assert ids[t].tolist() == full[:k].tolist()


def test_draft_topk_consistency_tiny_config():
    cfg = workloads.get_config(0)
    x = workloads.make_inputs(cfg, 0, "literal")
    d = oracle.draft_topk(x.hidden, x.w, x.bias, cfg.k)
    assert d["topk_id"].shape == (1, cfg.T, cfg.k)
    # the +1.5 blank bias dominates logits of sigma ~0.16: blank is top-1 of every slot
    assert (d["topk_id"][0, :, 0] == cfg.blank_id).all()
    assert np.all(np.diff(d["topk_logp"], axis=-1) <= 0)
    logp_full = d["z"] - d["lse"][..., None]
    assert np.allclose(np.take_along_axis(logp_full, d["topk_id"], -1), d["topk_logp"])
