"""Oracle: the Attention Draft Module's transformer layer (Sec. 3.1 "Model Structure": an attention draft
module takes the base model's last hidden states and predicts the draft positions with one transformer
layer whose construction is that of the base model; Sec. 3.3: its outputs go through the LM head).

Test infrastructure only (see the package docstring).

The paper gives the layer no formula of its own; it is the base family's decoder layer (Vicuna = LLaMA:
pre-normalisation with RMSNorm, multi-head attention with rotary position embeddings, gated SiLU feed-forward,
no biases), applied to the T draft positions in parallel over the layer's own key/value cache of the
history.  Everything is float64 and written out step by step.
"""
import numpy as np


def rms_norm(x, weight, eps):
    """Root-mean-square normalisation over the last axis: x / sqrt(mean(x^2) + eps) * weight."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(weight, dtype=np.float64)


def rope(x, pos, theta):
    """Rotary position embedding of one head vector x [dh] at integer position pos, half-split pairing:
    the pair (x[i], x[i + dh/2]) is rotated by the angle pos * theta^(-2i/dh)."""
    x = np.asarray(x, dtype=np.float64)
    dh = x.shape[-1]
    half = dh // 2
    out = np.empty_like(x)
    for i in range(half):
        ang = float(pos) * float(theta) ** (-2.0 * i / dh)
        cs, sn = np.cos(ang), np.sin(ang)
        a, b = x[i], x[i + half]
        out[i] = a * cs - b * sn
        out[i + half] = b * cs + a * sn
    return out


def silu(x):
    x = np.asarray(x, dtype=np.float64)
    return x / (1.0 + np.exp(-x))


def draft_layer_qkv(x, w, pos0, n_heads, eps, theta):
    """First half of the layer: normalised input -> queries, keys and values of the T new positions, queries
    and keys rotated to their positions pos0 .. pos0+T-1.  Returns (q [H, T, dh], k_new [H, T, dh],
    v_new [H, T, dh]) in float64; k_new and v_new are what the cache stores for these positions."""
    x = np.asarray(x, dtype=np.float64)
    T, D = x.shape
    H = n_heads
    dh = D // H
    h = rms_norm(x, w["ln1"], eps)
    q = (h @ np.asarray(w["wq"], dtype=np.float64).T).reshape(T, H, dh)
    k = (h @ np.asarray(w["wk"], dtype=np.float64).T).reshape(T, H, dh)
    v = (h @ np.asarray(w["wv"], dtype=np.float64).T).reshape(T, H, dh)
    q_rot = np.empty((H, T, dh))
    k_new = np.empty((H, T, dh))
    v_new = np.empty((H, T, dh))
    for t in range(T):
        for hd in range(H):
            q_rot[hd, t] = rope(q[t, hd], pos0 + t, theta)
            k_new[hd, t] = rope(k[t, hd], pos0 + t, theta)
            v_new[hd, t] = v[t, hd]
    return q_rot, k_new, v_new


def draft_layer_attend(x, w, q_rot, k_new, v_new, k_cache, v_cache, ctx_len, eps):
    """Second half: attention of the T new positions over the cached history and, causally, over each other,
    output projection and residual, then the gated feed-forward block and its residual.  Returns y [T, D]."""
    x = np.asarray(x, dtype=np.float64)
    T, D = x.shape
    q_rot = np.asarray(q_rot, dtype=np.float64)
    k_new = np.asarray(k_new, dtype=np.float64)
    v_new = np.asarray(v_new, dtype=np.float64)
    H, _, dh = q_rot.shape
    f = {k: np.asarray(v, dtype=np.float64) for k, v in w.items()}
    kc = np.asarray(k_cache, dtype=np.float64)
    vc = np.asarray(v_cache, dtype=np.float64)
    attn = np.empty((T, H, dh))
    scale = 1.0 / np.sqrt(dh)
    for hd in range(H):
        for t in range(T):
            # position t sees the whole cached history and the new positions up to itself
            keys = np.concatenate([kc[hd, :ctx_len], k_new[hd, : t + 1]], axis=0)
            vals = np.concatenate([vc[hd, :ctx_len], v_new[hd, : t + 1]], axis=0)
            s = keys @ q_rot[hd, t] * scale
            p = np.exp(s - s.max())
            p /= p.sum()
            attn[t, hd] = p @ vals
    h1 = x + attn.reshape(T, D) @ f["wo"].T
    m = rms_norm(h1, f["ln2"], eps)
    act = silu(m @ f["wg"].T) * (m @ f["wu"].T)
    return h1 + act @ f["wd"].T


def draft_layer(x, w, pos0, k_cache, v_cache, ctx_len, n_heads, eps, theta):
    """One sequence.  x [T, D]: the base model's hidden states at the T positions pos0 .. pos0+T-1.
    w: dict of float arrays - ln1 [D], wq, wk, wv, wo [D, D] (row = output feature; head h owns output rows
    h*dh .. h*dh+dh-1 of wq/wk/wv and input columns of wo), ln2 [D], wg, wu [F, D], wd [D, F].
    k_cache, v_cache [H, cap, dh]: keys (already rotated) and values of the ctx_len earlier positions.
    Returns (y [T, D], k_new [H, T, dh] rotated keys, v_new [H, T, dh]) in float64."""
    q_rot, k_new, v_new = draft_layer_qkv(x, w, pos0, n_heads, eps, theta)
    y = draft_layer_attend(x, w, q_rot, k_new, v_new, k_cache, v_cache, ctx_len, eps)
    return y, k_new, v_new
