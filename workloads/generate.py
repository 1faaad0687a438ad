"""Seeded input generation for the draft+verify step.  Inputs only: no method arithmetic.

Every tensor is drawn from numpy's PCG64 in the fixed order written in
`make_inputs`, in float32, and then rounded ONCE to the config's storage dtype
(bf16: round-to-nearest-even on the top 16 bits).  The returned float32 arrays
hold exactly the values the device sees, so a float64 consumer and a bf16
consumer start from identical numbers.
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

from .configs import StepConfig


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even.  NaN stays NaN."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    out = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float32 array to the storage dtype and return it as float32 again."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(x))
    raise ValueError(dtype)


@dataclass
class StepInputs:
    cfg: StepConfig
    seed: int
    variant: str
    hidden: np.ndarray       # [B,T,D] f32 (storage-rounded)
    w: np.ndarray            # [V+1,D] f32 (storage-rounded), row V is the blank
    bias: np.ndarray         # [V+1] f32, zero except the blank
    root_token: np.ndarray   # [B] i32
    q: np.ndarray            # [B,H,max_nodes,dh]
    k_tree: np.ndarray       # [B,H,max_nodes,dh]
    v_tree: np.ndarray       # [B,H,max_nodes,dh]
    k_cache: np.ndarray      # [B,H,kv_cap,dh]; rows >= ctx_len[b] are NaN (never to be used)
    v_cache: np.ndarray      # [B,H,kv_cap,dh]
    ctx_len: np.ndarray      # [B] i32
    kv_off: np.ndarray       # [B] i64 element offset of sequence b in the cache buffers
    proj: Optional[np.ndarray] = None  # [Vproj, H*dh] f32 verifier projection (tiny config only)
    planted: dict = field(default_factory=dict)  # structured variant: what was planted


def _rms_normalise(x: np.ndarray) -> np.ndarray:
    rms = np.sqrt(np.mean(x.astype(np.float64) ** 2, axis=-1, keepdims=True))
    return (x / rms).astype(np.float32)


def make_inputs(cfg: StepConfig, seed: int = 0, variant: str = "literal",
                with_attention: bool = True) -> StepInputs:
    """Draw one batch of step inputs.

    variant:
      "literal"    - the distributions the config states: hidden ~ N(0,1) (unit RMS per row when
                     cfg.rms_norm), W ~ N(0, 0.02^2), blank logit bias cfg.blank_bias.
      "ar1"        - as literal, but slot t's hidden state is 0.9*slot(t-1) + sqrt(1-0.81)*noise,
                     so neighbouring slots tend to share their top tokens (repeats occur).
      "structured" - peaky, blank-heavy, repeat-heavy posteriors such as a trained CTC head gives:
                     each slot's hidden state is a blend of a few planted head rows plus noise,
                     neighbouring slots share planted tokens, and the blank bias is raised so that
                     the blank lands inside most top-k sets.
    Draw order: W, hidden noise, (structured: plant choices), root_token, ctx_len, Q, K_tree, V_tree,
    K_cache, V_cache, proj.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    B, T, D, Vp1 = cfg.B, cfg.T, cfg.D, cfg.Vp1
    w = rng.standard_normal((Vp1, D), dtype=np.float32)
    w *= np.float32(0.02)
    w = round_to_storage(w, cfg.dtype)
    noise = rng.standard_normal((B, T, D), dtype=np.float32)
    bias = np.zeros(Vp1, dtype=np.float32)
    bias[cfg.blank_id] = np.float32(cfg.blank_bias)
    planted = {}
    if variant == "literal":
        hidden = noise
    elif variant == "ar1":
        hidden = noise.copy()
        rho = np.float32(0.9)
        for t in range(1, T):
            hidden[:, t] = rho * hidden[:, t - 1] + np.float32(np.sqrt(1.0 - 0.81)) * noise[:, t]
    elif variant == "structured":
        n_plant = 3
        coef = np.array([1.0, 0.8, 0.65], dtype=np.float32)
        tok = np.zeros((B, T, n_plant), dtype=np.int64)
        for b in range(B):
            for t in range(T):
                fresh = rng.integers(0, cfg.V, size=n_plant)
                if t > 0:
                    u = rng.random(n_plant)
                    # primary token repeats its predecessor half of the time; the runner-up is often
                    # the predecessor's primary token; otherwise new tokens
                    if u[0] < 0.5:
                        fresh[0] = tok[b, t - 1, 0]
                    if u[1] < 0.4 and tok[b, t - 1, 0] != fresh[0]:
                        fresh[1] = tok[b, t - 1, 0]
                    elif u[1] < 0.6 and tok[b, t - 1, 1] != fresh[0]:
                        fresh[1] = tok[b, t - 1, 1]
                # planted tokens of one slot must be distinct
                while len(set(fresh.tolist())) < n_plant:
                    fresh = np.where(np.arange(n_plant) == 0, fresh, rng.integers(0, cfg.V, size=n_plant))
                tok[b, t] = fresh
        direction = np.einsum("btpd,p->btd", w[tok], coef).astype(np.float32)
        direction = _rms_normalise(direction)
        alpha = np.float32(0.22 if cfg.rms_norm else 0.9)
        base = _rms_normalise(noise) if cfg.rms_norm else noise
        hidden = alpha * direction * (np.float32(1.0) if cfg.rms_norm else np.float32(8.0)) \
            + np.float32(np.sqrt(1.0 - float(alpha) ** 2)) * base
        # blank logit near the runner-up planted token so that it is inside most top-k sets
        plant_logit = np.einsum("btd,btpd->btp", hidden.astype(np.float64), w[tok].astype(np.float64))
        bias[cfg.blank_id] = np.float32(np.median(plant_logit[..., 1]))
        planted = {"tokens": tok, "blank_bias": float(bias[cfg.blank_id])}
    else:
        raise ValueError(variant)
    if cfg.rms_norm:
        hidden = _rms_normalise(hidden)
    hidden = round_to_storage(hidden, cfg.dtype)

    root_token = rng.integers(0, cfg.V, size=B).astype(np.int32)
    lo, hi = cfg.ctx
    ctx_len = rng.integers(lo, hi + 1, size=B).astype(np.int32)
    H, N, dh, cap = cfg.H, cfg.max_nodes, cfg.dh, cfg.kv_cap
    kv_off = (np.arange(B, dtype=np.int64) * (H * cap * dh)).astype(np.int64)
    if with_attention:
        q = round_to_storage(rng.standard_normal((B, H, N, dh), dtype=np.float32), cfg.dtype)
        k_tree = round_to_storage(rng.standard_normal((B, H, N, dh), dtype=np.float32), cfg.dtype)
        v_tree = round_to_storage(rng.standard_normal((B, H, N, dh), dtype=np.float32), cfg.dtype)
        k_cache = round_to_storage(rng.standard_normal((B, H, cap, dh), dtype=np.float32), cfg.dtype)
        v_cache = round_to_storage(rng.standard_normal((B, H, cap, dh), dtype=np.float32), cfg.dtype)
        for b in range(B):
            k_cache[b, :, ctx_len[b]:, :] = np.nan
            v_cache[b, :, ctx_len[b]:, :] = np.nan
    else:
        z = np.zeros((0,), dtype=np.float32)
        q = k_tree = v_tree = k_cache = v_cache = z
    proj = None
    if cfg.name == "tiny":
        proj = rng.standard_normal((cfg.V, H * dh), dtype=np.float32)
    return StepInputs(cfg=cfg, seed=seed, variant=variant, hidden=hidden, w=w, bias=bias,
                      root_token=root_token, q=q, k_tree=k_tree, v_tree=v_tree, k_cache=k_cache,
                      v_cache=v_cache, ctx_len=ctx_len, kv_off=kv_off, proj=proj, planted=planted)


@dataclass
class AttentionCase:
    """Operands of one verification-attention call (storage-rounded float32 arrays)."""
    q: np.ndarray         # [B,H,max_nodes,dh]
    k_tree: np.ndarray    # [B,H,max_nodes,dh]
    v_tree: np.ndarray    # [B,H,max_nodes,dh]
    k_cache: np.ndarray   # [B,H,kv_cap,dh]; rows >= ctx_len[b] are NaN
    v_cache: np.ndarray   # [B,H,kv_cap,dh]
    ctx_len: np.ndarray   # [B] i32
    kv_off: np.ndarray    # [B] i64
    kv_cap: int
    spiked: list          # per sequence: key positions (context rows, then ctx_len + node) that were scaled up


def make_attention_case(seed: int, B: int, H: int, max_nodes: int, dh: int, kv_cap: int, ctx_len,
                        dtype: str = "bf16", *, q_scale: float = 1.0, key_growth: float = 0.0,
                        n_spikes: int = 0, spike_scale: float = 12.0) -> AttentionCase:
    """Attention operands whose scores are NOT the flat N(0,1)-products of `make_inputs`: the peaked score
    distributions of a trained model, where the running maximum of a row keeps moving along the keys.

    q_scale     every query scaled (scores of standard deviation q_scale * sqrt(dh) before the 1/sqrt(dh))
    key_growth  key j of a sequence (context rows in order, then the tree nodes) scaled by 1 + key_growth * j / n_keys:
                later keys have the larger norm, so maxima tend to arrive late
    n_spikes    that many keys per sequence and head scaled by spike_scale; always among them: the last context row,
                a row of the context's last 32, the root's key and the deepest-numbered node's key, the rest uniform
                over all keys - large scores in late tiles and in every part of the key range
    Values N(0,1) throughout.  Draw order: Q, K_tree, V_tree, K_cache, V_cache, spike positions."""
    rng = np.random.Generator(np.random.PCG64(seed))
    ctx_len = np.broadcast_to(np.asarray(ctx_len, dtype=np.int32), (B,)).copy()
    q = rng.standard_normal((B, H, max_nodes, dh), dtype=np.float32) * np.float32(q_scale)
    k_tree = rng.standard_normal((B, H, max_nodes, dh), dtype=np.float32)
    v_tree = rng.standard_normal((B, H, max_nodes, dh), dtype=np.float32)
    k_cache = rng.standard_normal((B, H, kv_cap, dh), dtype=np.float32)
    v_cache = rng.standard_normal((B, H, kv_cap, dh), dtype=np.float32)
    spiked = []
    for b in range(B):
        L = int(ctx_len[b])
        n_keys = L + max_nodes
        if key_growth:
            ramp = (1.0 + key_growth * np.arange(n_keys, dtype=np.float32) / np.float32(n_keys)).astype(np.float32)
            k_cache[b, :, :L] *= ramp[None, :L, None]
            k_tree[b] *= ramp[None, L:, None]
        pos_b = []
        for h in range(H):
            forced = [L + 0, L + max_nodes - 1]
            if L > 0:
                forced += [L - 1, max(0, L - 1 - int(rng.integers(0, 32)))]
            pos = list(dict.fromkeys(forced))[:n_spikes]
            while len(pos) < n_spikes:
                j = int(rng.integers(0, n_keys))
                if j not in pos:
                    pos.append(j)
            for j in pos:
                if j < L:
                    k_cache[b, h, j] *= np.float32(spike_scale)
                else:
                    k_tree[b, h, j - L] *= np.float32(spike_scale)
            pos_b.append(pos)
        spiked.append(pos_b)
        k_cache[b, :, L:, :] = np.nan
        v_cache[b, :, L:, :] = np.nan
    kv_off = (np.arange(B, dtype=np.int64) * (H * kv_cap * dh)).astype(np.int64)
    return AttentionCase(q=round_to_storage(q, dtype), k_tree=round_to_storage(k_tree, dtype),
                         v_tree=round_to_storage(v_tree, dtype), k_cache=round_to_storage(k_cache, dtype),
                         v_cache=round_to_storage(v_cache, dtype), ctx_len=ctx_len, kv_off=kv_off, kv_cap=kv_cap,
                         spiked=spiked)


def make_topk_case(seed: int, B: int, T: int, k: int, blank_id: int, *, vocab: int = 12,
                   p_blank: float = 0.5, quantum: float = 0.0, first_blank: bool = False):
    """Synthetic per-slot top-k lists for exercising the collapse/tree stage directly.

    Token ids come from a small vocabulary so that neighbouring slots often share tokens; the blank is
    put into a slot's list with probability p_blank (always, and in first place, when first_blank).
    log-probabilities are negative, sorted descending per slot; quantum > 0 rounds them to multiples of
    `quantum` so that exact score ties occur.  Returns (topk_id [B,T,k] i32, topk_logp [B,T,k] f32).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    ids = np.zeros((B, T, k), dtype=np.int32)
    logp = np.zeros((B, T, k), dtype=np.float32)
    for b in range(B):
        for t in range(T):
            pool = rng.permutation(vocab)[:k].astype(np.int32)
            if first_blank:
                pool[0] = blank_id
            elif rng.random() < p_blank:
                pool[rng.integers(0, k)] = blank_id
            ids[b, t] = pool
            lp = -np.sort(rng.exponential(1.5, size=k)).astype(np.float32) - np.float32(0.05)
            if quantum > 0:
                lp = (np.round(lp / quantum) * quantum).astype(np.float32)
                lp = -np.sort(-lp)
            logp[b, t] = lp
    return ids, logp


@dataclass
class DraftLayerCase:
    """Inputs of one call of the draft module's transformer layer (storage-rounded float32 arrays)."""
    B: int
    T: int
    D: int
    H: int
    F: int
    kv_cap: int
    eps: float
    theta: float
    dtype: str
    x: np.ndarray          # [B,T,D] base-model hidden states of the T draft positions
    weights: dict          # ln1 [D], wq wk wv wo [D,D], ln2 [D], wg wu [F,D], wd [D,F]
    pos0: np.ndarray       # [B] i32 position of the first of the T tokens
    ctx_len: np.ndarray    # [B] i32 cached positions of the layer's own history
    kv_off: np.ndarray     # [B] i64 element offset of sequence b in the cache buffers
    k_cache: np.ndarray    # [B,H,kv_cap,dh]; rows >= ctx_len[b] are NaN
    v_cache: np.ndarray    # [B,H,kv_cap,dh]


def make_draft_layer_case(seed: int, B: int, T: int, D: int, H: int, F: int, ctx_len, kv_cap: int,
                          dtype: str = "bf16", eps: float = 1e-6, theta: float = 10000.0) -> DraftLayerCase:
    """Random decoder-layer weights at the scale of a trained LLaMA layer (projection entries about
    1/sqrt(fan_in), norm gains around 1), hidden states with a few large channels as the base model's last
    layer has, and a cache of unit-scale keys and values.  pos0 = ctx_len (the new tokens follow the history)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    dh = D // H
    ctx_len = np.broadcast_to(np.asarray(ctx_len, dtype=np.int32), (B,)).copy()

    def mat(rows, cols):
        return round_to_storage(rng.standard_normal((rows, cols), dtype=np.float32) / np.float32(np.sqrt(cols)), dtype)

    weights = {
        "ln1": round_to_storage(1.0 + 0.1 * rng.standard_normal(D, dtype=np.float32), dtype),
        "wq": mat(D, D), "wk": mat(D, D), "wv": mat(D, D), "wo": mat(D, D),
        "ln2": round_to_storage(1.0 + 0.1 * rng.standard_normal(D, dtype=np.float32), dtype),
        "wg": mat(F, D), "wu": mat(F, D), "wd": mat(D, F),
    }
    x = rng.standard_normal((B, T, D), dtype=np.float32)
    x[..., rng.integers(0, D, size=max(1, D // 256))] *= np.float32(8.0)  # a few outlier channels
    x = round_to_storage(x, dtype)
    k_cache = round_to_storage(rng.standard_normal((B, H, kv_cap, dh), dtype=np.float32), dtype)
    v_cache = round_to_storage(rng.standard_normal((B, H, kv_cap, dh), dtype=np.float32), dtype)
    for b in range(B):
        k_cache[b, :, ctx_len[b]:, :] = np.nan
        v_cache[b, :, ctx_len[b]:, :] = np.nan
    kv_off = (np.arange(B, dtype=np.int64) * H * kv_cap * dh)
    return DraftLayerCase(B=B, T=T, D=D, H=H, F=F, kv_cap=kv_cap, eps=eps, theta=theta, dtype=dtype, x=x,
                          weights=weights, pos0=ctx_len.copy(), ctx_len=ctx_len, kv_off=kv_off,
                          k_cache=k_cache, v_cache=v_cache)
