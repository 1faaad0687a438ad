"""GPU parity of ctc_raw_tree (the literal layout of Sec. 3.1) against the oracle, and its equivalence with the
collapsed tree under tree_verify_attn.

Everything the call writes is discrete (or a copy of an fp32 score): bit-exact when the oracle is fed the GPU's
top-k lists.  The attention outputs of a kept raw node and of the collapsed node it stands for come from the
same keys in another order: within 2e-3 (relative, RMS floor), in practice a few fp32 ulps.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_harness import cached_inputs, dev_f32, dev_i32, dev_i64, rel_err_rms_floor, to_device

pytestmark = pytest.mark.gpu
FIELDS = ("cand_tokens", "cand_len", "cand_score", "cand_leaf", "node_token", "node_parent", "node_depth",
          "node_removed")


@pytest.fixture(scope="module")
def pkg():
    import paper_2412_00061_amd as m
    m.load_library()
    return m


def _compare(res, ids, logp, root, blank, beam, max_nodes):
    g = {k: v.cpu().numpy() for k, v in res.items()}
    for b in range(ids.shape[0]):
        r = oracle.raw_tree(ids[b], logp[b], int(root[b]), blank, beam, max_nodes)
        assert int(g["n_cand"][b]) == r["n_cand"] and int(g["n_nodes"][b]) == r["n_nodes"]
        for name in FIELDS:
            assert np.array_equal(g[name][b], r[name]), (b, name)
        assert np.array_equal(g["anc_mask"][b].view(np.uint64), r["anc_mask"]), (b, "anc_mask")


@pytest.mark.parametrize("cfg_index,variant", [(0, "literal"), (0, "ar1"), (1, "literal"), (1, "structured"),
                                               (3, "ar1"), (4, "structured")])
def test_raw_tree_on_the_steps_lists(pkg, cfg_index, variant):
    cfg, x = workloads.get_config(cfg_index), cached_inputs(cfg_index, 0, variant)
    ctx = pkg.Context.for_config(cfg)
    s12 = pkg.ctc_draft_topk(ctx, to_device(x.hidden, cfg.dtype), to_device(x.w, cfg.dtype), dev_f32(x.bias), cfg.k)
    print(f"ctc_raw_tree cfg={cfg.name} variant={variant}", flush=True)
    res = pkg.ctc_raw_tree(ctx, s12["topk_id"], s12["topk_logp"], dev_i32(x.root_token), cfg.blank_id, cfg.beam,
                           cfg.max_nodes)
    torch.cuda.synchronize()
    _compare(res, s12["topk_id"].cpu().numpy(), s12["topk_logp"].cpu().numpy(), x.root_token, cfg.blank_id, cfg.beam,
             cfg.max_nodes)
    ctx.close()


@pytest.mark.parametrize("seed,B,T,k,beam,max_nodes,kw", [
    (1, 2, 8, 4, 128, 128, dict(p_blank=0.9)),
    (2, 3, 4, 2, 16, 12, dict(first_blank=True)),          # the cap cuts candidates short
    (3, 1, 8, 4, 64, 128, dict(quantum=0.25)),             # exact score ties: smaller index first
    (4, 4, 1, 8, 8, 8, dict()),                            # one slot
    (5, 2, 6, 3, 100, 40, dict(vocab=5, p_blank=0.7)),     # few distinct tokens: many repeats
])
def test_raw_tree_synthetic_lists(pkg, seed, B, T, k, beam, max_nodes, kw):
    blank = 11
    ids, logp = workloads.make_topk_case(seed, B, T, k, blank, **kw)
    root = np.arange(B, dtype=np.int32) + 3
    ctx = pkg.Context(max_batch=B, max_slots=8, max_topk=8, max_vocab_rows=64, max_nodes=128, max_heads=1,
                      max_head_dim=8)
    res = pkg.ctc_raw_tree(ctx, dev_i32(ids), dev_f32(logp), dev_i32(root), blank, beam, max_nodes)
    torch.cuda.synchronize()
    _compare(res, ids, logp, root, blank, beam, max_nodes)
    ctx.close()


def test_raw_layout_attention_equals_collapsed_layout(pkg):
    """tree_verify_attn over both layouts of the same top-k lists: every kept raw node gets the output of the
    collapsed node that stands for the same collapsed prefix (its Q, K, V rows are that node's)."""
    cfg, x = workloads.get_config(1), cached_inputs(1, 0, "structured")
    ctx = pkg.Context.for_config(cfg)
    N, H, dh = cfg.max_nodes, cfg.H, cfg.dh
    s12 = pkg.ctc_draft_topk(ctx, to_device(x.hidden, cfg.dtype), to_device(x.w, cfg.dtype), dev_f32(x.bias), cfg.k)
    root = dev_i32(x.root_token)
    col = pkg.ctc_collapse_tree(ctx, s12["topk_id"], s12["topk_logp"], root, cfg.blank_id, cfg.beam, N)
    raw = pkg.ctc_raw_tree(ctx, s12["topk_id"], s12["topk_logp"], root, cfg.blank_id, cfg.beam, N)
    torch.cuda.synchronize()
    c = {k: v.cpu().numpy()[0] for k, v in col.items()}
    r = {k: v.cpu().numpy()[0] for k, v in raw.items()}

    def paths(t):
        out = {}
        for i in range(int(t["n_nodes"])):
            p, j = [], i
            while j > 0:
                p.append(int(t["node_token"][j]))
                j = int(t["node_parent"][j])
            out[i] = list(reversed(p))
        return out

    node_of = {tuple(p): i for i, p in paths(c).items()}
    stands_for = np.zeros(N, dtype=np.int64)
    shared = []
    for i, p in paths(r).items():
        y = oracle.ctc_collapse(p, cfg.blank_id)
        if y in node_of:
            stands_for[i] = node_of[y]
            if i > 0 and not r["node_removed"][i]:
                shared.append(i)
    assert len(shared) >= 8
    q, kt, vt = (to_device(a, cfg.dtype) for a in (x.q, x.k_tree, x.v_tree))
    idx = torch.from_numpy(stands_for).cuda()
    kc, vc = to_device(x.k_cache, cfg.dtype), to_device(x.v_cache, cfg.dtype)
    off, ln = dev_i64(x.kv_off), dev_i32(x.ctx_len)
    scale = 1.0 / math.sqrt(dh)
    out_col = pkg.tree_verify_attn(ctx, q, kc, vc, off, ln, cfg.kv_cap, kt, vt, col["n_nodes"], col["anc_mask"], scale)
    out_raw = pkg.tree_verify_attn(ctx, q[:, :, idx].contiguous(), kc, vc, off, ln, cfg.kv_cap,
                                   kt[:, :, idx].contiguous(), vt[:, :, idx].contiguous(), raw["n_nodes"],
                                   raw["anc_mask"], scale)
    torch.cuda.synchronize()
    a, b = out_raw.cpu().numpy()[0][:, shared], out_col.cpu().numpy()[0][:, stands_for[shared]]
    assert rel_err_rms_floor(a, b) <= 2e-3
    # what the layout costs: nodes spent on removed positions
    assert int(r["n_nodes"]) == N and int((r["node_removed"][:N] == 1).sum()) > 0
    ctx.close()
