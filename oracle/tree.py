"""Oracle, token tree: prefix tree of the kept drafts under the base token, and its ancestor mask.

Test infrastructure only (see the package docstring).
"""
import numpy as np

from .collapse import alignment_ranks, alignment_scores_f32, collapse_candidates


def build_prefix_tree(cand_tokens, root_token, max_nodes):
    """Token tree whose root-to-node paths are the prefixes of the kept drafts (Sec. 2.1: draft
    tokens organised as a tree, paths from the root being candidate sequences; Sec. 3.3).

    Node 0 is the root and holds the base model's own greedy token (Sec. 3.3, the "base token"); the
    drafts hang below it.  Drafts are inserted in the given (rank) order, token by token; a node is
    created when the current node has no child with that token, and node ids are creation order.
    Once the tree holds max_nodes nodes nothing more is created: the draft being inserted keeps the
    prefix it already has, and later drafts still map onto existing nodes.

    Returns (node_token, node_parent, node_depth, cand_leaf) as Python lists; cand_leaf[c] is the node
    of draft c's last token, or -1 when the cap cut the draft short."""
    node_token, node_parent, node_depth = [int(root_token)], [-1], [0]
    cand_leaf = []
    for y in cand_tokens:
        cur, whole = 0, True
        for tok in y:
            child = -1
            for j in range(len(node_token)):
                if node_parent[j] == cur and node_token[j] == int(tok):
                    child = j
                    break
            if child < 0:
                if len(node_token) >= max_nodes:
                    whole = False
                    break
                node_token.append(int(tok))
                node_parent.append(cur)
                node_depth.append(node_depth[cur] + 1)
                child = len(node_token) - 1
            cur = child
        cand_leaf.append(cur if whole else -1)
    return node_token, node_parent, node_depth, cand_leaf


def ancestor_mask(node_parent):
    """Tree attention mask (Sec. 2.1, tree-structured verification; Sec. 3.1, positions of removed
    tokens are masked): mask[i, j] is True iff node j lies on the path from the root to node i,
    both ends included.  bool [N, N]."""
    n = len(node_parent)
    m = np.zeros((n, n), dtype=bool)
    for i in range(n):
        j = i
        while j >= 0:
            m[i, j] = True
            j = node_parent[j]
    return m


def pack_mask_u64(mask, max_nodes):
    """Bit-pack a bool [N, N] mask into uint64 [max_nodes, ceil(max_nodes/64)]: bit (j % 64) of word
    (j // 64) of row i is mask[i, j]; rows >= N are zero."""
    words = (max_nodes + 63) // 64
    out = np.zeros((max_nodes, words), dtype=np.uint64)
    n = mask.shape[0]
    for i in range(n):
        for j in range(n):
            if mask[i, j]:
                out[i, j // 64] |= np.uint64(1) << np.uint64(j % 64)
    return out


def collapse_tree(topk_id, topk_logp, root_token, blank, beam, max_nodes):
    """Stage 3 of the step for one sequence: drafts, prefix tree, ancestor mask, in the padded array
    layout the device library writes (integer pads -1, score pad -inf, length pad 0)."""
    ids = np.asarray(topk_id)
    T = ids.shape[0]
    drafts = collapse_candidates(ids, topk_logp, blank, beam)
    tok, par, dep, leaf = build_prefix_tree([d[0] for d in drafts], root_token, max_nodes)
    n_cand, n_nodes = len(drafts), len(tok)
    cand_tokens = np.full((beam, T), -1, dtype=np.int32)
    cand_len = np.zeros(beam, dtype=np.int32)
    cand_score = np.full(beam, -np.inf, dtype=np.float32)
    cand_leaf = np.full(beam, -1, dtype=np.int32)
    cand_rep = np.full(beam, -1, dtype=np.int64)
    for c, (y, s, idx) in enumerate(drafts):
        cand_tokens[c, :len(y)] = y
        cand_len[c] = len(y)
        cand_score[c] = s
        cand_leaf[c] = leaf[c]
        cand_rep[c] = idx
    node_token = np.full(max_nodes, -1, dtype=np.int32)
    node_parent = np.full(max_nodes, -1, dtype=np.int32)
    node_depth = np.full(max_nodes, -1, dtype=np.int32)
    node_token[:n_nodes], node_parent[:n_nodes], node_depth[:n_nodes] = tok, par, dep
    mask = ancestor_mask(par)
    return {
        "n_cand": n_cand, "cand_tokens": cand_tokens, "cand_len": cand_len, "cand_score": cand_score,
        "cand_leaf": cand_leaf, "cand_rep": cand_rep, "n_nodes": n_nodes, "node_token": node_token,
        "node_parent": node_parent, "node_depth": node_depth, "mask": mask,
        "anc_mask": pack_mask_u64(mask, max_nodes),
    }


def raw_tree(topk_id, topk_logp, root_token, blank, beam, max_nodes):
    """The layout Sec. 3.1 describes literally, for one sequence: the raw candidates keep their full length T
    (blanks and repeats included) and are combined in a token tree as they are; the CTC transform does not
    shorten them but marks the positions it removes - blanks, and tokens equal to the raw token right before
    them - and the attention map hides those positions from everything below them.

    Raw candidates are the k^T slot combinations valued by Eq. 6 (float32, left to right), ordered by
    (score descending, idx ascending); identical raw sequences (possible only when a slot's list names a
    token twice) count once, at their first place; the first `beam` are kept and inserted into a prefix tree over RAW
    tokens under the same node cap rule as the collapsed tree.  The first slot has no raw token before it
    (the root is the base model's token, not a draft slot).  mask[i, j]: j is i itself, or the root, or an
    ancestor of i that is not removed.

    Returns the padded arrays of collapse_tree plus node_removed (1 removed, 0 kept, -1 no node)."""
    ids = np.asarray(topk_id)
    T, k = ids.shape
    ranks = alignment_ranks(T, k)
    score = alignment_scores_f32(topk_logp, ranks)
    order, raws, seen = [], [], set()
    for i in sorted(range(ranks.shape[0]), key=lambda i: (-float(score[i]), i)):
        raw = tuple(int(ids[t, ranks[i, t]]) for t in range(T))
        if raw in seen:      # a list that names a token twice: the same raw sequence again, not a new candidate
            continue
        seen.add(raw)
        order.append(i)
        raws.append(raw)
        if len(raws) == beam:
            break
    tok, par, dep, leaf = build_prefix_tree(raws, root_token, max_nodes)
    n_cand, n_nodes = len(raws), len(tok)
    removed = [0] * n_nodes
    for i in range(1, n_nodes):
        repeat = dep[i] >= 2 and tok[i] == tok[par[i]]
        removed[i] = 1 if (tok[i] == blank or repeat) else 0
    mask = np.zeros((n_nodes, n_nodes), dtype=bool)
    for i in range(n_nodes):
        mask[i, i] = True
        j = par[i]
        while j >= 0:
            if not removed[j]:
                mask[i, j] = True
            j = par[j]
    cand_tokens = np.full((beam, T), -1, dtype=np.int32)
    cand_len = np.zeros(beam, dtype=np.int32)
    cand_score = np.full(beam, -np.inf, dtype=np.float32)
    cand_leaf = np.full(beam, -1, dtype=np.int32)
    for c, (raw, i) in enumerate(zip(raws, order)):
        cand_tokens[c], cand_len[c], cand_score[c], cand_leaf[c] = raw, T, score[i], leaf[c]
    node_token = np.full(max_nodes, -1, dtype=np.int32)
    node_parent = np.full(max_nodes, -1, dtype=np.int32)
    node_depth = np.full(max_nodes, -1, dtype=np.int32)
    node_removed = np.full(max_nodes, -1, dtype=np.int32)
    node_token[:n_nodes], node_parent[:n_nodes], node_depth[:n_nodes], node_removed[:n_nodes] = tok, par, dep, removed
    return {
        "n_cand": n_cand, "cand_tokens": cand_tokens, "cand_len": cand_len, "cand_score": cand_score,
        "cand_leaf": cand_leaf, "n_nodes": n_nodes, "node_token": node_token, "node_parent": node_parent,
        "node_depth": node_depth, "node_removed": node_removed, "mask": mask,
        "anc_mask": pack_mask_u64(mask, max_nodes),
    }
