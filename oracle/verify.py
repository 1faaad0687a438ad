"""Oracle, closing the step: the base model's greedy token after every tree node, and the update of the
decoding history (KV cache) with the accepted path.

Test infrastructure only (see the package docstring).
"""
import numpy as np


def verifier_head_argmax(node_hidden, w_base, n_nodes):
    """Greedy token of the base model after each tree node (Sec. 3.1: the base model ends in an LM head
    that maps hidden states to the vocabulary; Sec. 2.1: greedy decoding takes the most probable token).

    node_hidden [max_nodes, D]: last-layer hidden state of the base model at each tree node;
    w_base [V, D]: the base model's LM head (no blank row: the blank exists only in the draft head).
    Returns (z [max_nodes, V] float64 logits, target int32 [max_nodes]); target[i] = argmax_v z[i, v] for
    i < n_nodes, the smaller id among equal logits, and -1 for rows that hold no node."""
    h = np.asarray(node_hidden, dtype=np.float64)
    w = np.asarray(w_base, dtype=np.float64)
    z = h @ w.T
    target = np.full(h.shape[0], -1, dtype=np.int32)
    target[:n_nodes] = np.argmax(z[:n_nodes], axis=-1)  # numpy returns the first (smallest) index of a maximum
    return z, target


def argmax_rows(z, n_nodes):
    """argmax of given logits (any float dtype, compared as they are), smaller id among equals; -1 beyond
    n_nodes.  Used to chain the discrete decision on the kernel's own fp32 logits."""
    z = np.asarray(z)
    target = np.full(z.shape[0], -1, dtype=np.int32)
    target[:n_nodes] = np.argmax(z[:n_nodes], axis=-1)
    return target


def kv_commit(k_cache, v_cache, ctx_len, k_tree, v_tree, accept_len, accept_nodes):
    """History update after acceptance (Sec. 3.3: the decoding history is updated according to the
    output): the keys and values of the accepted path - the root, which is the base model's own token,
    and the accept_len accepted draft tokens - are appended to the cached context in path order.

    k_cache, v_cache [H, kv_cap, dh] (modified copies are returned); k_tree, v_tree [H, max_nodes, dh];
    accept_nodes [T+1] node ids of the path, root first.  Rows that would fall beyond kv_cap are dropped
    and the new length saturates at kv_cap.  Returns (k_cache, v_cache, new_ctx_len)."""
    kc, vc = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    cap = kc.shape[1]
    pos = int(ctx_len)
    for j in range(int(accept_len) + 1):
        node = int(accept_nodes[j])
        if pos + j < cap:
            kc[:, pos + j, :] = k_tree[:, node, :]
            vc[:, pos + j, :] = v_tree[:, node, :]
    return kc, vc, min(pos + int(accept_len) + 1, cap)
