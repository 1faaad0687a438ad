"""Oracle: sampling-based acceptance on the token tree (Sec. 2.1: the accept / re-sample rule of speculative
sampling; Sec. 3.3: the longest sequence that satisfies the criterion is the step's output).

Test infrastructure only (see the package docstring).

Sec. 2.1 states the rule for one drafted token x with draft distribution P' and target distribution P: accept x
with probability min(1, P(x) / P'(x)); on rejection drop the rest of the draft and draw the token from
norm(max(0, P - P')).  (The section prints the ratio the other way round; the re-sampling distribution it prints,
target minus draft, and the papers it cites fix the reading used here.)  The tree of this method is built
deterministically - top-k, combination, collapse - so the draft distribution behind a node's token is a point
mass on that token, and the siblings under a node are tried one after the other, each against what the rejections
before it left of the target distribution.  sec2_rule_distribution() takes these steps literally and returns the
exact distribution of the step's outcome.

With point-mass proposals that outcome has the target model's own distribution, and it can be realised with one
uniform random number per node: draw the target's token at the node by inverting its cumulative distribution; if
a child carries that token, move there, otherwise the drawn token ends the step.  That is greedy acceptance with
"the target's greedy token" replaced by "the target's sampled token"; sample_token(), sample_nodes() and
accept_sampled() are this procedure, and the CPU tests pin its exact outcome distribution to the one of the literal
rule.
"""
import numpy as np

from .accept import accept_longest


def target_probs(logits_row, temperature):
    """Softmax of one row of the target model's logits at the given temperature (> 0), float64."""
    z = np.asarray(logits_row, dtype=np.float64) / float(temperature)
    e = np.exp(z - z.max())
    return e / e.sum()


def sample_token(logits_row, u, temperature):
    """The token drawn from softmax(logits / temperature) by the uniform number u in [0, 1): the first token, in
    vocabulary order, whose cumulative probability exceeds u."""
    cum = np.cumsum(target_probs(logits_row, temperature))
    v = int(np.searchsorted(cum, float(u), side="right"))
    if v >= cum.shape[0]:  # u above the rounded total: the last token with any probability
        v = int(np.nonzero(np.diff(np.concatenate([[0.0], cum])) > 0)[0][-1])
    return v


def sample_nodes(logits, n_nodes, uniforms, temperature):
    """logits [N, V], uniforms [N] -> sampled target token per node, -1 for rows past n_nodes."""
    out = np.full(np.asarray(logits).shape[0], -1, dtype=np.int32)
    for i in range(int(n_nodes)):
        out[i] = sample_token(logits[i], uniforms[i], temperature)
    return out


def accept_sampled(node_token, node_parent, n_nodes, logits, uniforms, temperature, T):
    """One step's outcome under sampling-based acceptance: the target's token is drawn at every node, then the
    path is followed as in greedy acceptance.  Returns what accept_longest returns."""
    target = sample_nodes(logits, n_nodes, uniforms, temperature)
    return accept_longest(node_token, node_parent, n_nodes, target, T)


def _children(node_parent, n_nodes, u):
    return [j for j in range(1, int(n_nodes)) if node_parent[j] == u]


def sec2_rule_distribution(node_token, node_parent, n_nodes, probs):
    """Exact outcome distribution of the rule of Sec. 2.1 applied literally on the tree.  probs [N, V]: the target
    distribution after each node.  Returns {(last accepted node, next token): probability}.

    At a node, r starts as the target distribution.  For each child in node order, with token x and a point-mass
    draft distribution on x: accept with probability min(1, r(x) / 1); otherwise r becomes
    norm(max(0, r - pointmass(x))), which is r with x removed, renormalised.  When every child is rejected the
    next token is drawn from r."""
    out = {}

    def visit(u, weight):
        r = np.array(probs[u], dtype=np.float64)
        for c in _children(node_parent, n_nodes, u):
            x = int(node_token[c])
            a = min(1.0, r[x] / 1.0)
            if a > 0.0:
                visit(c, weight * a)
            weight = weight * (1.0 - a)
            if weight <= 0.0:
                return
            point = np.zeros_like(r)
            point[x] = 1.0
            r = np.maximum(0.0, r - point)
            r = r / r.sum()
        for v in np.nonzero(r > 0)[0]:
            out[(u, int(v))] = out.get((u, int(v)), 0.0) + weight * r[v]

    visit(0, 1.0)
    return out


def sample_and_match_distribution(node_token, node_parent, n_nodes, probs):
    """Exact outcome distribution of accept_sampled when the uniform numbers are independent: the set of u that
    draws token v at a node is an interval of length probs[node, v]."""
    out = {}

    def visit(u, weight):
        kids = {int(node_token[c]): c for c in _children(node_parent, n_nodes, u)}
        for v in np.nonzero(np.asarray(probs[u]) > 0)[0]:
            w = weight * float(probs[u][v])
            if int(v) in kids:
                visit(kids[int(v)], w)
            else:
                out[(u, int(v))] = out.get((u, int(v)), 0.0) + w

    visit(0, 1.0)
    return out
