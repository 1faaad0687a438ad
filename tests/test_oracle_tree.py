"""Pins for the oracle's prefix tree and ancestor mask.  CPU only."""
import numpy as np
import pytest

import oracle
import workloads


def _trie_by_nested_dicts(cands, max_nodes):
    """Independent route: a dict-of-dicts trie; ids handed out in creation order."""
    root = {"id": 0, "kids": {}}
    count = 1
    created = [(None, -1, 0)]  # (token, parent, depth) per id; root token filled by caller
    leaves = []
    for y in cands:
        node, depth, whole = root, 0, True
        for tok in y:
            depth += 1
            if tok not in node["kids"]:
                if count >= max_nodes:
                    whole = False
                    break
                node["kids"][tok] = {"id": count, "kids": {}}
                created.append((tok, node["id"], depth))
                count += 1
            node = node["kids"][tok]
        leaves.append(node["id"] if whole else -1)
    return created, leaves


def _random_cands(rng, n, T, vocab):
    seen, out = set(), []
    while len(out) < n:
        y = tuple(rng.integers(0, vocab, size=rng.integers(1, T + 1)).tolist())
        if y not in seen:
            seen.add(y)
            out.append(y)
    return out


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("max_nodes", [1, 2, 7, 20, 128])
def test_tree_matches_nested_dict_trie(seed, max_nodes):
    rng = np.random.Generator(np.random.PCG64(seed))
    cands = _random_cands(rng, 25, 5, 3)
    tok, par, dep, leaf = oracle.build_prefix_tree(cands, 77, max_nodes)
    created, leaves = _trie_by_nested_dicts(cands, max_nodes)
    assert tok[0] == 77 and par[0] == -1 and dep[0] == 0
    assert [(t, p, d) for t, p, d in zip(tok[1:], par[1:], dep[1:])] == created[1:]
    assert leaf == leaves
    assert len(tok) <= max_nodes


def _path_tokens(tok, par, i):
    out = []
    while i > 0:
        out.append(tok[i])
        i = par[i]
    return tuple(reversed(out))


@pytest.mark.parametrize("seed", range(6))
def test_tree_invariants(seed):
    rng = np.random.Generator(np.random.PCG64(50 + seed))
    T = 6
    cands = _random_cands(rng, 30, T, 3)
    cap = [128, 40, 9][seed % 3]
    tok, par, dep, leaf = oracle.build_prefix_tree(cands, 5, cap)
    n = len(tok)
    assert n <= cap
    prefixes = {y[:d] for y in cands for d in range(1, len(y) + 1)}
    if cap == 128:
        assert n == 1 + len(prefixes)  # one node per distinct non-empty prefix
    kids = set()
    for i in range(1, n):
        assert 0 <= par[i] < i and dep[i] == dep[par[i]] + 1 <= T
        assert (par[i], tok[i]) not in kids  # sibling tokens distinct
        kids.add((par[i], tok[i]))
        assert _path_tokens(tok, par, i) in prefixes
    for y, lf in zip(cands, leaf):
        if lf >= 0:
            assert _path_tokens(tok, par, lf) == y
        else:
            assert n == cap
    mask = oracle.ancestor_mask(par)
    assert mask.shape == (n, n)
    assert not np.triu(mask, 1).any()  # a node only sees earlier-created nodes and itself
    for i in range(n):
        assert mask[i, i] and mask[i, 0]
        assert mask[i].sum() == dep[i] + 1
        if i:
            expect = mask[par[i]].copy()
            expect[i] = True
            assert np.array_equal(mask[i], expect)


def test_child_may_repeat_parent_token_and_no_blank_enters():
    # a _ a collapses to (a, a): the tree must hold a child with its parent's token
    blank = 9
    ids = np.array([[4, blank], [blank, 4], [4, blank]])
    logp = np.array([[-0.1, -2.0], [-0.2, -1.0], [-0.1, -3.0]], dtype=np.float32)
    r = oracle.collapse_tree(ids, logp, 1, blank, 8, 16)
    cands = [tuple(row[:l]) for row, l in zip(r["cand_tokens"].tolist(), r["cand_len"].tolist()) if l]
    assert (4, 4) in cands and (4,) in cands
    n = r["n_nodes"]
    assert blank not in r["node_token"][:n].tolist()
    two = [i for i in range(n) if r["node_depth"][i] == 2]
    assert any(r["node_token"][i] == r["node_token"][r["node_parent"][i]] for i in two)


def test_cap_keeps_prefix_and_later_candidates_still_map():
    cands = [(1, 2, 3), (1, 2), (4,), (1,)]
    tok, par, dep, leaf = oracle.build_prefix_tree(cands, 0, 3)  # root + 2 nodes only
    assert tok == [0, 1, 2] and par == [-1, 0, 1] and dep == [0, 1, 2]
    assert leaf == [-1, 2, -1, 1]
    tok, par, dep, leaf = oracle.build_prefix_tree(cands, 0, 1)
    assert tok == [0] and leaf == [-1, -1, -1, -1]


def test_pack_mask_bits():
    par = [-1, 0, 1, 0] + [3] * 70
    mask = oracle.ancestor_mask(par)
    packed = oracle.pack_mask_u64(mask, 128)
    assert packed.shape == (128, 2) and packed.dtype == np.uint64
    for i in range(128):
        for j in range(128):
            bit = (int(packed[i, j // 64]) >> (j % 64)) & 1
            want = bool(mask[i, j]) if i < len(par) and j < len(par) else False
            assert bool(bit) == want
    assert int(packed[70, 1]) == 1 << (70 - 64) and int(packed[70, 0]) == 0b1001


def test_collapse_tree_layout_tiny_config():
    cfg = workloads.get_config(0)
    x = workloads.make_inputs(cfg, 0, "ar1")
    d = oracle.draft_topk(x.hidden[0], x.w, x.bias, cfg.k)
    r = oracle.collapse_tree(d["topk_id"], d["topk_logp"].astype(np.float32), int(x.root_token[0]),
                             cfg.blank_id, cfg.beam, cfg.max_nodes)
    nc, n = r["n_cand"], r["n_nodes"]
    assert 1 <= nc <= cfg.beam and 1 < n <= cfg.max_nodes
    assert (r["cand_tokens"][nc:] == -1).all() and (r["cand_len"][nc:] == 0).all()
    assert np.isneginf(r["cand_score"][nc:]).all() and (r["cand_leaf"][nc:] == -1).all()
    assert (r["node_token"][n:] == -1).all() and (r["node_parent"][n:] == -1).all()
    assert np.all(np.diff(r["cand_score"][:nc]) <= 0)
    assert r["node_token"][0] == x.root_token[0]
    assert (r["anc_mask"][n:] == 0).all()
