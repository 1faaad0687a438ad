"""Pins for the oracle's tree-masked verification attention.  CPU only."""
import numpy as np
import pytest

import oracle


def _textbook_causal_attention(q, k, v, scale):
    """Plain causal self-attention over one sequence, written with a full score matrix.
    q, k, v [S, dh] -> [S, dh]."""
    s = scale * (q @ k.T)
    s = np.where(np.tril(np.ones_like(s, dtype=bool)), s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=1, keepdims=True)
    return p @ v


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def test_chain_tree_is_causal_attention():
    rng = np.random.Generator(np.random.PCG64(0))
    H, L, N, dh = 3, 11, 6, 8
    q, kt, vt = _rand(rng, H, N, dh), _rand(rng, H, N, dh), _rand(rng, H, N, dh)
    kc, vc = _rand(rng, H, L + 2, dh), _rand(rng, H, L + 2, dh)
    parent = [-1] + list(range(N - 1))
    mask = oracle.ancestor_mask(parent)
    out = oracle.tree_attention(q, kc, vc, L, kt, vt, N, mask, 0.3)
    for h in range(H):
        k_all = np.concatenate([kc[h, :L], kt[h]])
        v_all = np.concatenate([vc[h, :L], vt[h]])
        q_all = np.concatenate([np.zeros((L, dh)), q[h]])
        ref = _textbook_causal_attention(q_all, k_all, v_all, 0.3)[L:]
        assert np.allclose(out[h], ref, rtol=1e-12, atol=1e-12)


def test_single_node_tree_is_decode_attention():
    rng = np.random.Generator(np.random.PCG64(1))
    H, L, dh = 2, 9, 4
    q, kt, vt = _rand(rng, H, 1, dh), _rand(rng, H, 1, dh), _rand(rng, H, 1, dh)
    kc, vc = _rand(rng, H, L, dh), _rand(rng, H, L, dh)
    out = oracle.tree_attention(q, kc, vc, L, kt, vt, 1, np.ones((1, 1), bool), 0.5)
    for h in range(H):
        keys = np.concatenate([kc[h], kt[h]])
        vals = np.concatenate([vc[h], vt[h]])
        logits = 0.5 * keys @ q[h, 0]
        w = np.exp(logits - np.logaddexp.reduce(logits))
        assert np.allclose(out[h, 0], w @ vals, rtol=1e-12, atol=1e-12)


def test_star_tree_sees_context_root_and_self_only():
    rng = np.random.Generator(np.random.PCG64(2))
    H, L, N, dh = 1, 5, 5, 4
    q, kt, vt = _rand(rng, H, N, dh), _rand(rng, H, N, dh), _rand(rng, H, N, dh)
    kc, vc = _rand(rng, H, L, dh), _rand(rng, H, L, dh)
    mask = oracle.ancestor_mask([-1, 0, 0, 0, 0])
    out = oracle.tree_attention(q, kc, vc, L, kt, vt, N, mask, 1.0)
    for i in range(1, N):
        keys = np.concatenate([kc[0], kt[0, [0, i]]])
        vals = np.concatenate([vc[0], vt[0, [0, i]]])
        s = keys @ q[0, i]
        w = np.exp(s - s.max())
        assert np.allclose(out[0, i], (w / w.sum()) @ vals, rtol=1e-12, atol=1e-12)
    # changing a sibling's key/value must not change node 1
    kt2, vt2 = kt.copy(), vt.copy()
    kt2[0, 2:] += 3.0
    vt2[0, 2:] -= 5.0
    out2 = oracle.tree_attention(q, kc, vc, L, kt2, vt2, N, mask, 1.0)
    assert np.array_equal(out[0, 1], out2[0, 1])


def test_each_node_equals_attention_over_its_own_path():
    # the defining property of tree verification: node i's output is what ordinary causal attention
    # would give for the sequence context + root path of i
    rng = np.random.Generator(np.random.PCG64(3))
    H, L, dh = 2, 7, 8
    parent = [-1, 0, 0, 1, 1, 2, 3, 3, 5, 6]
    N = len(parent)
    q, kt, vt = _rand(rng, H, N + 3, dh), _rand(rng, H, N + 3, dh), _rand(rng, H, N + 3, dh)
    kc, vc = _rand(rng, H, L, dh), _rand(rng, H, L, dh)
    mask = oracle.ancestor_mask(parent)
    out = oracle.tree_attention(q, kc, vc, L, kt, vt, N, mask, 0.35)
    assert out.shape == (H, N, dh)
    for i in range(N):
        path = []
        j = i
        while j >= 0:
            path.append(j)
            j = parent[j]
        path.reverse()
        for h in range(H):
            k_all = np.concatenate([kc[h], kt[h, path]])
            v_all = np.concatenate([vc[h], vt[h, path]])
            q_all = np.concatenate([np.zeros((L, dh)), q[h, path]])
            ref = _textbook_causal_attention(q_all, k_all, v_all, 0.35)[-1]
            assert np.allclose(out[h, i], ref, rtol=1e-12, atol=1e-12)


def test_context_length_zero_and_rows_beyond_ctx_ignored():
    rng = np.random.Generator(np.random.PCG64(4))
    H, N, dh = 1, 3, 4
    q, kt, vt = _rand(rng, H, N, dh), _rand(rng, H, N, dh), _rand(rng, H, N, dh)
    kc = np.full((H, 4, dh), np.nan)
    vc = np.full((H, 4, dh), np.nan)
    mask = oracle.ancestor_mask([-1, 0, 1])
    out = oracle.tree_attention(q, kc, vc, 0, kt, vt, N, mask, 1.0)
    assert np.isfinite(out).all()
    assert np.allclose(out[0, 0], vt[0, 0])  # the root alone: weight 1 on itself


def test_holes_in_raw_tree_equal_collapsed_tree():
    """The paper keeps raw candidates at full length and masks the positions the CTC transform removed
    (Sec. 3.1); this build collapses first and attends over the deduplicated tree.  Both give every
    surviving token the same visible set, hence the same output: checked for every raw candidate of a
    small case, with K/V/Q of a raw position determined by the collapsed prefix it stands for."""
    rng = np.random.Generator(np.random.PCG64(5))
    blank, T, k, L, dh = 0, 4, 2, 6, 8
    ids = np.array([[1, blank], [1, 2], [blank, 2], [2, 3]])
    logp = -rng.random((T, k)).astype(np.float32)
    r = oracle.collapse_tree(ids, logp, 7, blank, 1000, 128)
    n = r["n_nodes"]
    q, kt, vt = _rand(rng, 1, n, dh), _rand(rng, 1, n, dh), _rand(rng, 1, n, dh)
    kc, vc = _rand(rng, 1, L, dh), _rand(rng, 1, L, dh)
    out = oracle.tree_attention(q, kc, vc, L, kt, vt, n, r["mask"], 0.4)
    node_of = {}
    for i in range(n):
        path, j = [], i
        while j > 0:
            path.append(int(r["node_token"][j]))
            j = int(r["node_parent"][j])
        node_of[tuple(reversed(path))] = i
    checked = 0
    for rk in oracle.alignment_ranks(T, k):
        raw = [int(ids[t, rk[t]]) for t in range(T)]
        kept = [t for t in range(T) if raw[t] != blank and (t == 0 or raw[t] != raw[t - 1])]
        for pos, t in enumerate(kept):
            # raw layout: the token at slot t sees context, root and the kept slots before it
            prefix_nodes = [0] + [node_of[tuple(raw[u] for u in kept[:p + 1])] for p in range(pos + 1)]
            me = prefix_nodes[-1]
            keys = np.concatenate([kc[0], kt[0, prefix_nodes]])
            vals = np.concatenate([vc[0], vt[0, prefix_nodes]])
            s = 0.4 * keys @ q[0, me]
            w = np.exp(s - s.max())
            assert np.allclose(out[0, me], (w / w.sum()) @ vals, rtol=1e-12, atol=1e-12)
            checked += 1
    assert checked > 20
