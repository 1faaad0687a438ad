"""Oracle, greedy acceptance: the longest drafted path the base model agrees with.

Test infrastructure only (see the package docstring).
"""
import numpy as np


def verifier_argmax(attn_out, proj):
    """Stand-in for the base model's greedy token after each tree node: the argmax over the
    vocabulary of a fixed random projection of the node's attention output (all heads
    concatenated).  attn_out [H, n, dh], proj [V, H*dh].  Equal values -> smaller id.  int32 [n]."""
    o = np.asarray(attn_out, dtype=np.float64)
    H, n, dh = o.shape
    flat = o.transpose(1, 0, 2).reshape(n, H * dh)
    return np.argmax(flat @ np.asarray(proj, dtype=np.float64).T, axis=-1).astype(np.int32)


def accept_longest(node_token, node_parent, n_nodes, target, T):
    """Greedy acceptance (Sec. 2.1: accept what matches the target model's greedy output; Sec. 3.3:
    the longest sequence that satisfies the criterion is this step's output).

    target[i] is the base model's greedy token after node i.  Starting at the root, move to the child
    whose token equals target[current]; stop when no child matches.  Returns
    (accept_len, accept_nodes [T+1], accept_tokens [T+1], next_token): accept_len counts accepted
    draft tokens (the root, the base model's own token, is always part of the output and not
    counted), the arrays list the path root first padded with -1, and next_token is target at the
    last accepted node."""
    cur, length = 0, 0
    path = [0]
    while True:
        nxt = -1
        for j in range(1, int(n_nodes)):
            if node_parent[j] == cur and node_token[j] == target[cur]:
                nxt = j
                break
        if nxt < 0:
            break
        cur = nxt
        length += 1
        path.append(cur)
    nodes = np.full(T + 1, -1, dtype=np.int32)
    toks = np.full(T + 1, -1, dtype=np.int32)
    nodes[:len(path)] = path
    toks[:len(path)] = [node_token[j] for j in path]
    return length, nodes, toks, int(target[cur])
