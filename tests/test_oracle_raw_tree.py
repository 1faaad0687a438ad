"""CPU pins of the literal (fixed-length, masked) tree layout of Sec. 3.1: a hand case, the visible set of every
node against the collapse rule (pinned on its own), the node cap, and the equivalence with the collapsed tree
under attention."""
import numpy as np

import oracle

A, B_, C, BLANK = 5, 6, 9, 0


def _one_candidate(raw, root=3):
    """Top-k lists whose single combination is `raw` (k = 1)."""
    ids = np.array([[t] for t in raw])
    logp = np.full((len(raw), 1), -0.5, dtype=np.float32)
    return oracle.raw_tree(ids, logp, root, BLANK, 4, 32)


def test_hand_case_a_a_blank_b():
    r = _one_candidate([A, A, BLANK, B_])
    assert r["n_nodes"] == 5 and list(r["node_token"][:5]) == [3, A, A, BLANK, B_]
    assert list(r["node_removed"][:5]) == [0, 0, 1, 1, 0]  # the repeat and the blank
    m = r["mask"]
    assert list(np.flatnonzero(m[4])) == [0, 1, 4]      # b sees root, the first a, itself
    assert list(np.flatnonzero(m[2])) == [0, 1, 2]      # a removed position still sees its own prefix
    assert list(np.flatnonzero(m[3])) == [0, 1, 3]
    assert list(r["cand_tokens"][0]) == [A, A, BLANK, B_] and r["cand_len"][0] == 4 and r["cand_leaf"][0] == 4


def test_repeat_after_a_blank_is_kept_and_the_root_is_no_slot():
    r = _one_candidate([A, BLANK, A, A], root=A)
    # first a: no raw token before it (the root's token equals it, but the root is not a slot)
    assert list(r["node_removed"][:5]) == [0, 0, 1, 0, 1]
    assert list(np.flatnonzero(r["mask"][3])) == [0, 1, 3]


def _case(seed, T, k, vocab):
    rng = np.random.default_rng(seed)
    ids = np.stack([rng.permutation(vocab)[:k] + 1 for _ in range(T)])  # tokens 1..vocab, each once per list
    ids[rng.integers(0, T), rng.integers(0, k)] = BLANK
    logp = -np.sort(rng.exponential(1.0, size=(T, k)).astype(np.float32), axis=-1)
    return ids, logp


def test_visible_tokens_are_the_collapsed_prefix():
    """For every node: the tokens it sees below the root, in path order and without itself when it is removed,
    are exactly the collapse of its raw prefix."""
    for seed, T, k, vocab in [(0, 4, 3, 4), (1, 5, 2, 3), (2, 6, 2, 3)]:
        ids, logp = _case(seed, T, k, vocab)
        r = oracle.raw_tree(ids, logp, 7, BLANK, k ** T, 4096)
        n, tok, par = r["n_nodes"], r["node_token"], r["node_parent"]
        assert r["n_cand"] == k ** T and np.all(r["cand_leaf"][:k ** T] > 0)
        for i in range(1, n):
            path, j = [], i
            while j > 0:
                path.append(j)
                j = par[j]
            path.reverse()
            raw_prefix = [int(tok[j]) for j in path]
            seen = [int(tok[j]) for j in path if r["mask"][i, j] and not (j == i and r["node_removed"][i])]
            assert tuple(seen) == oracle.ctc_collapse(raw_prefix, BLANK), (raw_prefix, seen)
            assert r["mask"][i, 0] and r["mask"][i, i]
            assert bool(r["node_removed"][i]) == (oracle.ctc_collapse(raw_prefix, BLANK) ==
                                                  oracle.ctc_collapse(raw_prefix[:-1], BLANK))


def test_order_and_node_cap():
    ids, logp = _case(3, 4, 3, 5)
    full = oracle.raw_tree(ids, logp, 1, BLANK, 81, 4096)
    s = full["cand_score"][:81]
    assert np.all(s[:-1] >= s[1:])
    capped = oracle.raw_tree(ids, logp, 1, BLANK, 81, 10)
    assert capped["n_nodes"] == 10 and np.array_equal(capped["node_token"][:10], full["node_token"][:10])
    assert np.any(capped["cand_leaf"][:81] == -1) and capped["cand_leaf"][0] == full["cand_leaf"][0]
    assert np.all(capped["node_removed"][10:] == -1)


def test_attention_over_the_raw_tree_equals_the_collapsed_tree():
    """Every surviving raw node stands for a collapsed prefix; with the keys, values and queries of that prefix
    its attention output over the raw layout equals the collapsed tree's output at the prefix's node."""
    rng = np.random.default_rng(9)
    T, k, L, dh = 4, 2, 5, 8
    ids = np.array([[1, BLANK], [1, 2], [BLANK, 2], [2, 3]])
    logp = -rng.random((T, k)).astype(np.float32)
    col = oracle.collapse_tree(ids, logp, 7, BLANK, 1000, 256)
    raw = oracle.raw_tree(ids, logp, 7, BLANK, 1000, 256)
    nc, nr = col["n_nodes"], raw["n_nodes"]
    node_of = {(): 0}
    for i in range(1, nc):
        path, j = [], i
        while j > 0:
            path.append(int(col["node_token"][j]))
            j = int(col["node_parent"][j])
        node_of[tuple(reversed(path))] = i
    stands_for = np.zeros(nr, dtype=np.int64)  # collapsed node of each raw node's collapsed prefix
    for i in range(1, nr):
        path, j = [], i
        while j > 0:
            path.append(int(raw["node_token"][j]))
            j = int(raw["node_parent"][j])
        stands_for[i] = node_of[oracle.ctc_collapse(list(reversed(path)), BLANK)]
    q, kt, vt = (rng.standard_normal((1, nc, dh)) for _ in range(3))
    kc, vc = rng.standard_normal((1, L, dh)), rng.standard_normal((1, L, dh))
    out_col = oracle.tree_attention(q, kc, vc, L, kt, vt, nc, col["mask"], 0.4)
    out_raw = oracle.tree_attention(q[:, stands_for], kc, vc, L, kt[:, stands_for], vt[:, stands_for], nr,
                                    raw["mask"], 0.4)
    kept = [i for i in range(1, nr) if not raw["node_removed"][i]]
    assert len(kept) > 10
    for i in kept:
        assert np.allclose(out_raw[0, i], out_col[0, stands_for[i]], rtol=1e-12, atol=1e-12)
    assert nr > nc  # the raw layout spends nodes on removed positions


def test_a_token_named_twice_in_a_list_gives_one_candidate():
    ids = np.array([[A, A], [B_, BLANK]])
    logp = np.array([[-0.1, -0.3], [-0.2, -0.4]], dtype=np.float32)
    r = oracle.raw_tree(ids, logp, 1, BLANK, 8, 16)
    assert r["n_cand"] == 2 and [list(t) for t in r["cand_tokens"][:2]] == [[A, B_], [A, BLANK]]
    assert np.allclose(r["cand_score"][:2], [-0.3, -0.5])  # the better of the two equal sequences
