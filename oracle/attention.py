"""Oracle, verification attention of the base model over the token tree.

Test infrastructure only (see the package docstring).  float64 throughout.
"""
import numpy as np


def tree_attention(q, k_cache, v_cache, ctx_len, k_tree, v_tree, n_nodes, mask, scale):
    """One attention layer of the parallel verification pass (Sec. 2.1 tree verification, Sec. 3.3:
    all candidates are verified by the base model in one pass) for one sequence.

    q, k_tree, v_tree [H, >=n_nodes, dh]; k_cache, v_cache [H, >=ctx_len, dh]; mask bool
    [n_nodes, n_nodes] (ancestor-or-self).  Node i attends to the ctx_len cached positions (all of
    them) and to the tree nodes j with mask[i, j]; weights are softmax(scale * q_i . k) over exactly
    those keys.  Returns float64 [H, n_nodes, dh]."""
    q = np.asarray(q, dtype=np.float64)
    kc = np.asarray(k_cache, dtype=np.float64)
    vc = np.asarray(v_cache, dtype=np.float64)
    kt = np.asarray(k_tree, dtype=np.float64)
    vt = np.asarray(v_tree, dtype=np.float64)
    H, dh = q.shape[0], q.shape[-1]
    L, n = int(ctx_len), int(n_nodes)
    out = np.zeros((H, n, dh), dtype=np.float64)
    for h in range(H):
        for i in range(n):
            vis = np.nonzero(mask[i, :n])[0]
            keys = np.concatenate([kc[h, :L], kt[h, vis]], axis=0)
            vals = np.concatenate([vc[h, :L], vt[h, vis]], axis=0)
            s = scale * (keys @ q[h, i])
            p = np.exp(s - s.max())
            p /= p.sum()
            out[h, i] = p @ vals
    return out
