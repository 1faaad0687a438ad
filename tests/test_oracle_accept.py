"""Pins for the oracle's greedy acceptance and the verifier stand-in.  CPU only."""
import numpy as np
import pytest

import oracle
import workloads


def _tree(seed, beam=24, cap=64):
    ids, logp = workloads.make_topk_case(seed, 1, 6, 3, 99, vocab=6, p_blank=0.5)
    return oracle.collapse_tree(ids[0], logp[0], 42, 99, beam, cap)


def _brute_force_accept(r, target):
    """Longest kept draft prefix all of whose tokens equal the target at their parent node,
    found by trying every draft and every length."""
    tok, par = r["node_token"], r["node_parent"]
    best = [0]
    for i in range(r["n_nodes"]):
        path, j = [], i
        while j >= 0:
            path.append(j)
            j = int(par[j])
        path.reverse()
        if all(tok[path[d + 1]] == target[path[d]] for d in range(len(path) - 1)) and len(path) > len(best):
            best = path
    return best


@pytest.mark.parametrize("seed", range(10))
def test_planted_paths_are_recovered(seed):
    r = _tree(seed)
    n, T = r["n_nodes"], 6
    rng = np.random.Generator(np.random.PCG64(seed))
    for node in rng.integers(0, n, size=8):
        path, j = [], int(node)
        while j >= 0:
            path.append(j)
            j = int(r["node_parent"][j])
        path.reverse()
        target = np.full(n, 7777, dtype=np.int32)  # a token no node carries
        for a, b in zip(path[:-1], path[1:]):
            target[a] = r["node_token"][b]
        length, nodes, toks, nxt = oracle.accept_longest(r["node_token"], r["node_parent"], n, target, T)
        assert length == len(path) - 1 == r["node_depth"][node]
        assert nodes[:length + 1].tolist() == path and (nodes[length + 1:] == -1).all()
        assert toks[:length + 1].tolist() == [int(r["node_token"][j]) for j in path]
        assert nxt == 7777 and toks[0] == 42


@pytest.mark.parametrize("seed", range(10))
def test_random_targets_match_brute_force(seed):
    r = _tree(seed)
    n = r["n_nodes"]
    rng = np.random.Generator(np.random.PCG64(1000 + seed))
    for _ in range(20):
        target = rng.integers(0, 6, size=n).astype(np.int32)  # small vocabulary: frequent matches
        length, nodes, toks, nxt = oracle.accept_longest(r["node_token"], r["node_parent"], n, target, 6)
        best = _brute_force_accept(r, target)
        assert nodes[:length + 1].tolist() == best
        assert nxt == target[best[-1]]


def test_root_only_tree():
    length, nodes, toks, nxt = oracle.accept_longest([5], [-1], 1, [9], 4)
    assert length == 0 and nodes.tolist() == [0, -1, -1, -1, -1] and toks[0] == 5 and nxt == 9


def test_verifier_argmax_layout_and_ties():
    H, n, dh, V = 2, 3, 2, 5
    o = np.zeros((H, n, dh))
    o[0, 1, 1] = 1.0   # node 1: feature index 0*dh+1
    o[1, 2, 0] = 1.0   # node 2: feature index 1*dh+0
    proj = np.zeros((V, H * dh))
    proj[3, 1] = 2.0
    proj[4, 2] = 2.0
    t = oracle.verifier_argmax(o, proj)
    assert t.tolist() == [0, 3, 4]  # node 0: all scores equal -> smallest id
