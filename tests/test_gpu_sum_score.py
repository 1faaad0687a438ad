"""GPU parity of ctc_sum_score (Eq. 5 value of the candidate drafts) against the oracle.

The sums are compared with the oracle's float64 recursion run on the very fp32 logits and lse the GPU produced
(chained parity, as for the other stages): fp32 log-space arithmetic over T steps accumulates a few 1e-5 plus a
few ulps of the result's magnitude.  The rank order is decided on the kernel's own fp32 sums and must then match
bit for bit, ties to the smaller index.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_harness import cached_inputs, dev_f32, dev_i32, to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pkg():
    import paper_2412_00061_amd as m
    m.load_library()
    return m


def _tol(ref):
    return 2e-5 + 16 * np.spacing(np.abs(ref).astype(np.float32)).astype(np.float64)


def _check(pkg, cfg, x):
    ctx = pkg.Context.for_config(cfg)
    s12 = pkg.ctc_draft_topk(ctx, to_device(x.hidden, cfg.dtype), to_device(x.w, cfg.dtype), dev_f32(x.bias), cfg.k,
                             want_logits=True)
    s3 = pkg.ctc_collapse_tree(ctx, s12["topk_id"], s12["topk_logp"], dev_i32(x.root_token), cfg.blank_id, cfg.beam,
                               cfg.max_nodes)
    print(f"ctc_sum_score cfg={cfg.name} B={cfg.B} T={cfg.T} beam={cfg.beam}", flush=True)
    res = pkg.ctc_sum_score(ctx, s12["logits"], s12["lse"], s3["cand_tokens"], s3["cand_len"], s3["n_cand"],
                            cfg.blank_id)
    torch.cuda.synchronize()
    z, lse = s12["logits"].cpu().numpy(), s12["lse"].cpu().numpy()
    toks, lens, n_cand = (s3[k].cpu().numpy() for k in ("cand_tokens", "cand_len", "n_cand"))
    best = s3["cand_score"].cpu().numpy()
    got, rank = res["cand_logp_sum"].cpu().numpy(), res["cand_rank_sum"].cpu().numpy()
    for b in range(cfg.B):
        n = int(n_cand[b])
        ref = oracle.sum_scores(z[b], lse[b], toks[b], lens[b], n, cfg.blank_id)
        assert np.all(np.abs(got[b, :n] - ref[:n]) <= _tol(ref[:n])), np.max(np.abs(got[b, :n] - ref[:n]))
        assert np.all(np.isneginf(got[b, n:]))
        assert np.array_equal(rank[b], oracle.ranks_desc(got[b], n))
        # the best alignment (Eq. 6, what ctc_collapse_tree ranks by) is one term of the sum
        assert np.all(got[b, :n] >= best[b, :n] - 1e-4)
    ctx.close()
    return got, n_cand


@pytest.mark.parametrize("cfg_index,variant", [(0, "literal"), (0, "ar1"), (1, "literal"), (1, "structured"),
                                               (4, "ar1")])
def test_sum_score_on_the_steps_candidates(pkg, cfg_index, variant):
    _check(pkg, workloads.get_config(cfg_index), cached_inputs(cfg_index, 0, variant))


def test_sum_score_hand_case_and_edges(pkg):
    """Three slots, vocabulary {0, 1} + blank 2: the drafts (0), (0, 0), (0, 1), () and one too long for T."""
    T, Vp1, beam, blank = 3, 3, 8, 2
    rng = np.random.default_rng(5)
    logits = rng.standard_normal((1, T, Vp1)).astype(np.float32)
    lse = np.log(np.exp(logits.astype(np.float64)).sum(-1)).astype(np.float32)
    toks = np.full((1, beam, T), -1, dtype=np.int32)
    lens = np.zeros((1, beam), dtype=np.int32)
    drafts = [(0,), (0, 0), (0, 1), (), (0, 1, 0), (1, 1, 1)]
    for i, y in enumerate(drafts):
        toks[0, i, :len(y)], lens[0, i] = y, len(y)
    ctx = pkg.Context(max_batch=1, max_slots=8, max_topk=4, max_vocab_rows=8, max_nodes=8, max_heads=1, max_head_dim=8)
    res = pkg.ctc_sum_score(ctx, dev_f32(logits), dev_f32(lse), dev_i32(toks), dev_i32(lens),
                            dev_i32(np.array([len(drafts)], dtype=np.int32)), blank)
    torch.cuda.synchronize()
    got = res["cand_logp_sum"].cpu().numpy()[0]
    logp = logits[0].astype(np.float64) - lse[0].astype(np.float64)[:, None]
    for i, y in enumerate(drafts):
        ref = oracle.ctc_sequence_logprob(logp, y, blank)
        if np.isneginf(ref):
            assert np.isneginf(got[i]), (y, got[i])   # (1, 1, 1) needs five slots
        else:
            assert abs(got[i] - ref) <= 2e-5, (y, got[i], ref)
    assert np.all(np.isneginf(got[len(drafts):]))
    assert np.array_equal(res["cand_rank_sum"].cpu().numpy()[0], oracle.ranks_desc(got, len(drafts)))
    ctx.close()


def test_sum_score_and_raw_tree_reject_bad_arguments(pkg):
    ctx = pkg.Context(max_batch=1, max_slots=8, max_topk=8, max_vocab_rows=8, max_nodes=8, max_heads=1, max_head_dim=8)
    logits, lse = dev_f32(np.zeros((1, 3, 4), dtype=np.float32)), dev_f32(np.zeros((1, 3), dtype=np.float32))
    toks, lens = dev_i32(np.zeros((1, 4, 3), dtype=np.int32)), dev_i32(np.zeros((1, 4), dtype=np.int32))
    n = dev_i32(np.array([1], dtype=np.int32))
    with pytest.raises(pkg.CtcspecError, match="blank_id"):
        pkg.ctc_sum_score(ctx, logits, lse, toks, lens, n, 4)
    two = dev_f32(np.zeros((2, 3, 4), dtype=np.float32))
    with pytest.raises(pkg.CtcspecError, match="limits"):
        pkg.ctc_sum_score(ctx, two, dev_f32(np.zeros((2, 3), dtype=np.float32)), dev_i32(np.zeros((2, 4, 3), dtype=np.int32)),
                          dev_i32(np.zeros((2, 4), dtype=np.int32)), dev_i32(np.array([1, 1], dtype=np.int32)), 3)
    ids = dev_i32(np.zeros((1, 8, 8), dtype=np.int32))
    with pytest.raises(pkg.CtcspecError, match="exceeds"):  # 8^8 raw candidates
        pkg.ctc_raw_tree(ctx, ids, dev_f32(np.zeros((1, 8, 8), dtype=np.float32)), n, 0, 4, 8)
    with pytest.raises(pkg.CtcspecError, match="max_nodes"):
        pkg.ctc_raw_tree(ctx, dev_i32(np.zeros((1, 2, 2), dtype=np.int32)), dev_f32(np.zeros((1, 2, 2), dtype=np.float32)),
                         n, 0, 4, 500)
    ctx.close()
