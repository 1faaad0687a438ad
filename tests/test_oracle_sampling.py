"""Pins of the sampling-acceptance oracle (Sec. 2.1 rule on the tree of Sec. 3.3).

* the literal accept / re-sample rule with point-mass proposals and the one-uniform-per-node procedure have the same
  exact outcome distribution, and that distribution is the target model's own: P(first emitted token = v) = p_root(v);
* the draw itself: the set of uniform numbers that gives token v is the interval [C(v-1), C(v)) of the cumulative
  distribution (checked at both ends of every interval), temperature -> 0 gives the greedy token, and a hand case;
* accept_sampled with uniforms that select the greedy token everywhere is greedy acceptance.
"""
import numpy as np

import oracle


def _random_tree(rng, n, V):
    """A prefix tree of n nodes with sibling tokens distinct, the root's token arbitrary."""
    token = np.zeros(n, dtype=np.int32)
    parent = np.full(n, -1, dtype=np.int32)
    token[0] = rng.integers(0, V)
    used = {0: set()}
    for j in range(1, n):
        while True:
            p = int(rng.integers(0, j))
            free = [v for v in range(V) if v not in used[p]]
            if free:
                break
        parent[j] = p
        token[j] = rng.choice(free)
        used[p].add(int(token[j]))
        used[j] = set()
    return token, parent


def test_sec2_rule_equals_sample_and_match_and_is_the_target_distribution():
    rng = np.random.default_rng(0)
    for trial in range(40):
        V = int(rng.integers(2, 7))
        n = int(rng.integers(1, 9))
        token, parent = _random_tree(rng, n, V)
        probs = rng.dirichlet(np.full(V, 0.7), size=n)
        if trial % 4 == 0:  # some impossible tokens, some certain ones
            probs[rng.integers(0, n)] = np.eye(V)[rng.integers(0, V)]
        lit = oracle.sec2_rule_distribution(token, parent, n, probs)
        sam = oracle.sample_and_match_distribution(token, parent, n, probs)
        assert abs(sum(lit.values()) - 1.0) < 1e-12 and abs(sum(sam.values()) - 1.0) < 1e-12
        for key in set(lit) | set(sam):
            assert abs(lit.get(key, 0.0) - sam.get(key, 0.0)) < 1e-12, (trial, key)
        # the first token the step emits after the root: a child's token when the walk moves on, else the drawn one
        first = np.zeros(V)
        for (node, nxt), w in lit.items():
            cur = node
            while cur != 0 and parent[cur] != 0:
                cur = parent[cur]
            first[int(token[cur]) if node != 0 else nxt] += w
        assert np.allclose(first, probs[0], atol=1e-12), trial


def test_sample_token_inverts_the_cumulative_distribution():
    rng = np.random.default_rng(1)
    for V, temp in [(2, 1.0), (5, 0.7), (17, 1.3), (200, 1.0)]:
        z = rng.standard_normal(V) * 3.0
        p = np.exp(z / temp - np.max(z / temp))
        p /= p.sum()
        cum = np.cumsum(p)
        lo = 0.0
        for v in range(V):
            hi = cum[v]
            width = hi - lo
            if width > 1e-9:
                assert oracle.sample_token(z, lo + width * 1e-6, temp) == v
                assert oracle.sample_token(z, hi - width * 1e-6, temp) == v
            lo = hi
        assert oracle.sample_token(z, 0.0, temp) == 0
        assert np.allclose(oracle.target_probs(z, temp), p)


def test_sample_token_hand_case_and_cold_limit():
    z = np.log(np.array([0.5, 0.25, 0.125, 0.125]))
    assert [oracle.sample_token(z, u, 1.0) for u in (0.0, 0.49, 0.5, 0.74, 0.75, 0.874, 0.875, 0.999)] == [0, 0, 1, 1, 2, 2, 3, 3]
    # temperature 1/2 squares the probabilities: (16, 4, 1, 1) / 22
    assert [oracle.sample_token(z, u, 0.5) for u in (0.72, 0.73, 0.90, 0.91, 0.954, 0.956)] == [0, 1, 1, 2, 2, 3]
    rng = np.random.default_rng(2)
    for _ in range(20):
        row = rng.standard_normal(50)
        assert oracle.sample_token(row, rng.random(), 1e-3) == int(np.argmax(row))
    # a token with zero probability is never drawn
    assert oracle.sample_token(np.array([-np.inf, 0.0, -np.inf]), 0.0, 1.0) == 1
    assert oracle.sample_token(np.array([0.0, 0.0, -np.inf]), 0.999999, 1.0) == 1


def test_accept_sampled_reduces_to_greedy_when_the_draw_is_the_greedy_token():
    rng = np.random.default_rng(3)
    for _ in range(10):
        V, n, T = 9, 7, 4
        token, parent = _random_tree(rng, n, V)
        logits = rng.standard_normal((n, V)) * 2.0
        greedy = logits.argmax(-1)
        # a uniform in the middle of the greedy token's interval at every node
        u = np.empty(n)
        for i in range(n):
            cum = np.cumsum(oracle.target_probs(logits[i], 1.0))
            g = int(greedy[i])
            u[i] = ((cum[g - 1] if g else 0.0) + cum[g]) / 2.0
        got = oracle.accept_sampled(token, parent, n, logits, u, 1.0, T)
        ref = oracle.accept_longest(token, parent, n, greedy, T)
        assert got[0] == ref[0] and got[3] == ref[3]
        assert np.array_equal(got[1], ref[1]) and np.array_equal(got[2], ref[2])
        assert np.array_equal(oracle.sample_nodes(logits, n - 2, u, 1.0)[n - 2:], [-1, -1])
