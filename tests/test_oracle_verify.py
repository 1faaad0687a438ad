"""Pins for the oracle's verifier head (greedy token per tree node) and history update.  CPU only."""
import numpy as np
import pytest

import oracle


def test_argmax_of_a_selector_head_is_known_in_closed_form():
    # w_base = rows of a scaled identity: z[i, v] = c_v * h[i, v], so the greedy token of a one-hot hidden
    # state e_j is j, and of -e_j any other row with the largest (zero) logit: the smallest id != j
    D = V = 12
    w = np.diag(np.arange(1, V + 1, dtype=np.float64))
    h = np.zeros((8, D))
    for i in range(6):
        h[i, (5 * i) % D] = 1.0
    h[6, 0] = -1.0   # logits: -1 at 0, 0 elsewhere -> ties among 1..11 -> 1
    h[7, 3] = -2.0   # ties among all but 3 -> 0
    z, t = oracle.verifier_head_argmax(h, w, 8)
    assert t.tolist() == [0, 5, 10, 3, 8, 1, 1, 0]
    assert z.shape == (8, V) and z[1, 5] == 6.0


def test_argmax_matches_exhaustive_scan_with_ties():
    rng = np.random.Generator(np.random.PCG64(3))
    h = rng.integers(-2, 3, size=(40, 7)).astype(np.float64)
    w = rng.integers(-2, 3, size=(50, 7)).astype(np.float64)   # small integers: many exact ties
    z, t = oracle.verifier_head_argmax(h, w, 33)
    ties = 0
    for i in range(40):
        if i >= 33:
            assert t[i] == -1
            continue
        best, best_v = None, -1
        for v in range(50):
            s = sum(h[i, d] * w[v, d] for d in range(7))
            if best is None or s > best:
                best, best_v = s, v
        ties += int(np.sum(z[i] == best) > 1)
        assert t[i] == best_v
    assert ties > 5   # the case really exercises the tie rule
    assert np.array_equal(oracle.argmax_rows(z.astype(np.float32), 33), t)


def test_argmax_is_invariant_under_positive_scaling_and_row_permutation():
    rng = np.random.Generator(np.random.PCG64(4))
    h = rng.standard_normal((9, 16))
    w = rng.standard_normal((30, 16))
    _, t = oracle.verifier_head_argmax(h, w, 9)
    _, t2 = oracle.verifier_head_argmax(3.5 * h, w, 9)
    assert np.array_equal(t, t2)
    perm = rng.permutation(30)
    _, t3 = oracle.verifier_head_argmax(h, w[perm], 9)
    assert np.array_equal(perm[t3], t)


def _case(seed, H=3, cap=20, dh=4, N=10):
    rng = np.random.Generator(np.random.PCG64(seed))
    kc, vc = rng.standard_normal((H, cap, dh)), rng.standard_normal((H, cap, dh))
    kt, vt = rng.standard_normal((H, N, dh)), rng.standard_normal((H, N, dh))
    return kc, vc, kt, vt


def test_kv_commit_hand_case():
    kc, vc, kt, vt = _case(0)
    nodes = np.array([0, 4, 7, -1, -1], dtype=np.int32)
    k2, v2, new_len = oracle.kv_commit(kc, vc, 11, kt, vt, 2, nodes)
    assert new_len == 14
    for j, node in enumerate([0, 4, 7]):
        assert np.array_equal(k2[:, 11 + j], kt[:, node]) and np.array_equal(v2[:, 11 + j], vt[:, node])
    untouched = np.ones(20, dtype=bool)
    untouched[11:14] = False
    assert np.array_equal(k2[:, untouched], kc[:, untouched]) and np.array_equal(v2[:, untouched], vc[:, untouched])
    assert not np.shares_memory(k2, kc)


def test_kv_commit_root_only_and_saturation():
    kc, vc, kt, vt = _case(1)
    k2, v2, new_len = oracle.kv_commit(kc, vc, 5, kt, vt, 0, np.array([0, -1, -1], dtype=np.int32))
    assert new_len == 6 and np.array_equal(k2[:, 5], kt[:, 0])
    assert np.array_equal(np.delete(k2, 5, axis=1), np.delete(kc, 5, axis=1))
    # the path does not fit: rows beyond the capacity are dropped, the length saturates
    k3, v3, new_len = oracle.kv_commit(kc, vc, 18, kt, vt, 3, np.array([0, 2, 3, 9], dtype=np.int32))
    assert new_len == 20
    assert np.array_equal(k3[:, 18], kt[:, 0]) and np.array_equal(k3[:, 19], kt[:, 2])
    assert np.array_equal(k3[:, :18], kc[:, :18])


@pytest.mark.parametrize("seed", range(5))
def test_attention_over_committed_history_equals_attention_over_history_plus_path(seed):
    """What the update is for: a later query that attends the grown cache sees exactly the old context plus
    the accepted path - the same result as tree attention of a node whose ancestors are that path."""
    H, cap, dh, N = 2, 24, 8, 9
    rng = np.random.Generator(np.random.PCG64(100 + seed))
    kc, vc = rng.standard_normal((H, cap, dh)), rng.standard_normal((H, cap, dh))
    kt, vt = rng.standard_normal((H, N, dh)), rng.standard_normal((H, N, dh))
    q = rng.standard_normal((H, N, dh))
    L = 10
    path = [0, 3, 5]   # node 5 under node 3 under the root
    mask = np.zeros((N, N), dtype=bool)
    mask[5, path] = True
    mask[0, 0] = True
    scale = 1.0 / np.sqrt(dh)
    want = oracle.tree_attention(q, kc, vc, L, kt, vt, N, mask, scale)[:, 5]
    k2, v2, L2 = oracle.kv_commit(kc, vc, L, kt, vt, 2, np.array(path + [-1], dtype=np.int32))
    assert L2 == 13
    # the same query against the committed cache alone (a one-node "tree" that sees only itself is avoided
    # by giving the node an empty tree: plain softmax over the cache rows)
    for h in range(H):
        s = (k2[h, :L2] @ q[h, 5]) * scale
        w = np.exp(s - s.max())
        w /= w.sum()
        assert np.allclose(w @ v2[h, :L2], want[h], rtol=1e-12, atol=1e-12)
