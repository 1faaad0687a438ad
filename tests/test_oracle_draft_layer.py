"""CPU pins of the draft-module layer oracle (Sec. 3.1: one transformer layer of the base model's
construction).  Each pin is something other than the oracle's own formula: hand values, closed forms,
invariants of the rotary embedding, torch's library routines on CPU, and the equivalence of parallel and
one-token-at-a-time evaluation."""
import math

import numpy as np
import pytest
import torch

import oracle
from workloads import make_draft_layer_case


def _case(seed=0, B=1, T=4, D=32, H=4, F=48, ctx=5, cap=16):
    return make_draft_layer_case(seed, B, T, D, H, F, ctx, cap, dtype="f32")


def _run(c, b=0, **over):
    w = dict(c.weights)
    w.update(over)
    return oracle.draft_layer(c.x[b], w, int(c.pos0[b]), c.k_cache[b], c.v_cache[b], int(c.ctx_len[b]), c.H,
                              c.eps, c.theta)


def test_rms_norm_hand_values():
    # x = (3, 4): mean square 12.5
    y = oracle.rms_norm(np.array([3.0, 4.0]), np.array([1.0, 2.0]), 0.0)
    assert np.allclose(y, [3 / math.sqrt(12.5), 8 / math.sqrt(12.5)], rtol=1e-15)
    # scale invariance without eps, and eps only matters near zero
    x = np.array([0.5, -2.0, 1.5, 3.0])
    assert np.allclose(oracle.rms_norm(7.0 * x, np.ones(4), 0.0), oracle.rms_norm(x, np.ones(4), 0.0), rtol=1e-14)
    assert np.allclose(oracle.rms_norm(np.zeros(4), np.ones(4), 1e-6), 0.0)


def test_rope_is_the_plane_rotation():
    # dh = 2: one pair, angle = pos (frequency theta^0 = 1)
    y = oracle.rope(np.array([1.0, 0.0]), 3, 10000.0)
    assert np.allclose(y, [math.cos(3.0), math.sin(3.0)], rtol=1e-15)
    # dh = 4: pairs (0,2) and (1,3), the second at frequency theta^(-1/2)
    x = np.array([1.0, 2.0, 0.0, 0.0])
    y = oracle.rope(x, 5, 100.0)
    assert np.allclose(y, [math.cos(5.0), 2 * math.cos(0.5), math.sin(5.0), 2 * math.sin(0.5)], rtol=1e-14)
    # position 0 is the identity
    v = np.linspace(-1, 1, 8)
    assert np.array_equal(oracle.rope(v, 0, 10000.0), v)


def test_rope_preserves_norm_and_relative_position():
    rng = np.random.default_rng(1)
    q, k = rng.standard_normal(16), rng.standard_normal(16)
    for m, n in [(3, 1), (10, 8), (107, 105)]:
        assert math.isclose(np.linalg.norm(oracle.rope(q, m, 1e4)), np.linalg.norm(q), rel_tol=1e-13)
    d1 = oracle.rope(q, 3, 1e4) @ oracle.rope(k, 1, 1e4)
    d2 = oracle.rope(q, 10, 1e4) @ oracle.rope(k, 8, 1e4)
    d3 = oracle.rope(q, 107, 1e4) @ oracle.rope(k, 105, 1e4)
    assert math.isclose(d1, d2, rel_tol=1e-11) and math.isclose(d1, d3, rel_tol=1e-10)
    assert not math.isclose(d1, oracle.rope(q, 3, 1e4) @ oracle.rope(k, 2, 1e4), rel_tol=1e-3)


def test_silu_values():
    assert oracle.silu(0.0) == 0.0
    assert math.isclose(float(oracle.silu(1.0)), 1.0 / (1.0 + math.exp(-1.0)), rel_tol=1e-15)
    assert math.isclose(float(oracle.silu(30.0)), 30.0, rel_tol=1e-12)
    assert abs(float(oracle.silu(-30.0))) < 1e-11


def test_zero_output_projections_leave_the_residual_stream():
    c = _case()
    y, k_new, v_new = _run(c, wo=np.zeros_like(c.weights["wo"]), wd=np.zeros_like(c.weights["wd"]))
    assert np.array_equal(y, c.x[0].astype(np.float64))
    # keys keep their norm under the rotation: |k_new| = |h wk^T| per head
    h = oracle.rms_norm(c.x[0], c.weights["ln1"], c.eps)
    kk = (h @ c.weights["wk"].astype(np.float64).T).reshape(c.T, c.H, -1)
    assert np.allclose(np.linalg.norm(k_new, axis=-1), np.linalg.norm(kk, axis=-1).T, rtol=1e-12)
    vv = (h @ c.weights["wv"].astype(np.float64).T).reshape(c.T, c.H, -1)
    assert np.allclose(v_new, vv.transpose(1, 0, 2), rtol=1e-13)


def test_uniform_attention_closed_form():
    """Zero queries make every score 0, so attention is the plain average of the visible values: with the
    cached values all equal to one ramp per head and the new values zero (wv = 0), position t returns the
    ramp scaled by ctx / (ctx + t + 1)."""
    c = _case(seed=3)
    D, H = c.D, c.H
    dh = D // H
    zero = np.zeros((D, D), dtype=np.float32)
    w = dict(c.weights, wq=zero, wv=zero, wd=np.zeros_like(c.weights["wd"]))
    vc = np.broadcast_to(np.arange(dh, dtype=np.float32), c.v_cache[0].shape).copy()
    ctx = int(c.ctx_len[0])
    y, _, _ = oracle.draft_layer(c.x[0], w, int(c.pos0[0]), c.k_cache[0], vc, ctx, H, c.eps, c.theta)
    for t in range(c.T):
        mix = np.tile(np.arange(dh, dtype=np.float64) * ctx / (ctx + t + 1), H)
        assert np.allclose(y[t], c.x[0, t] + mix @ w["wo"].astype(np.float64).T, rtol=1e-12, atol=1e-12)


def test_causality_and_history_dependence():
    c = _case(seed=4)
    y, k_new, _ = _run(c)
    x2 = c.x.copy()
    x2[0, 2] += 1.0  # a later position changes...
    y2, k2, _ = oracle.draft_layer(x2[0], c.weights, int(c.pos0[0]), c.k_cache[0], c.v_cache[0], int(c.ctx_len[0]),
                                   c.H, c.eps, c.theta)
    assert np.array_equal(y[:2], y2[:2]) and not np.allclose(y[2:], y2[2:])  # ...nothing before it
    kc = c.k_cache.copy()
    kc[0, :, 0, :] *= -1.0  # the history matters to every position
    y3, _, _ = oracle.draft_layer(c.x[0], c.weights, int(c.pos0[0]), kc[0], c.v_cache[0], int(c.ctx_len[0]), c.H,
                                  c.eps, c.theta)
    assert not np.allclose(y, y3)
    # rows of the cache beyond ctx_len are never read (they hold NaN)
    assert np.isfinite(y).all() and np.isnan(c.k_cache[0, :, int(c.ctx_len[0]):]).all()


def test_parallel_equals_one_token_at_a_time():
    """T positions in one call = T calls of one position each, the cache growing by the new key and value."""
    c = _case(seed=5, T=5, ctx=3, cap=12)
    y, k_new, v_new = _run(c)
    kc, vc = c.k_cache[0].astype(np.float64).copy(), c.v_cache[0].astype(np.float64).copy()
    ctx = int(c.ctx_len[0])
    for t in range(c.T):
        yt, kt, vt = oracle.draft_layer(c.x[0, t:t + 1], c.weights, int(c.pos0[0]) + t, kc, vc, ctx, c.H, c.eps, c.theta)
        assert np.allclose(yt[0], y[t], rtol=1e-11, atol=1e-12)
        kc[:, ctx], vc[:, ctx] = kt[:, 0], vt[:, 0]
        ctx += 1
    assert np.allclose(kc[:, int(c.ctx_len[0]):ctx], k_new, rtol=1e-12)


def _torch_layer(c, b=0):
    """The same layer from torch's library routines (linear, scaled_dot_product_attention, silu), float64."""
    F = torch.nn.functional
    tw = {k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in c.weights.items()}
    x = torch.from_numpy(c.x[b].astype(np.float64))
    T, D, H = c.T, c.D, c.H
    dh = D // H
    ctx = int(c.ctx_len[b])

    def norm(v, g):
        return v * torch.rsqrt(v.pow(2).mean(-1, keepdim=True) + c.eps) * g

    def rot(v, pos):  # v [T, H, dh], complex multiplication on the (i, i + dh/2) pairs
        half = dh // 2
        freqs = torch.pow(torch.tensor(c.theta, dtype=torch.float64), -torch.arange(half, dtype=torch.float64) * 2 / dh)
        ang = pos[:, None].double() * freqs[None]
        z = torch.complex(v[..., :half], v[..., half:]) * torch.polar(torch.ones_like(ang), ang)[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    h = norm(x, tw["ln1"])
    pos = torch.arange(T) + int(c.pos0[b])
    q = rot(F.linear(h, tw["wq"]).view(T, H, dh), pos).transpose(0, 1)
    k = rot(F.linear(h, tw["wk"]).view(T, H, dh), pos).transpose(0, 1)
    v = F.linear(h, tw["wv"]).view(T, H, dh).transpose(0, 1)
    keys = torch.cat([torch.from_numpy(c.k_cache[b, :, :ctx].astype(np.float64)), k], dim=1)
    vals = torch.cat([torch.from_numpy(c.v_cache[b, :, :ctx].astype(np.float64)), v], dim=1)
    mask = torch.ones(T, ctx + T, dtype=torch.bool)
    mask[:, ctx:] = torch.tril(torch.ones(T, T, dtype=torch.bool))
    a = F.scaled_dot_product_attention(q, keys, vals, attn_mask=mask)  # default scale 1/sqrt(dh)
    h1 = x + F.linear(a.transpose(0, 1).reshape(T, D), tw["wo"])
    m = norm(h1, tw["ln2"])
    y = h1 + F.linear(F.silu(F.linear(m, tw["wg"])) * F.linear(m, tw["wu"]), tw["wd"])
    return y.numpy(), k.numpy(), v.numpy()


@pytest.mark.parametrize("seed,T,D,H,F,ctx", [(0, 4, 32, 4, 48, 5), (1, 8, 64, 2, 96, 0), (2, 1, 32, 8, 40, 11)])
def test_against_torch_library_routines(seed, T, D, H, F, ctx):
    c = make_draft_layer_case(seed, 2, T, D, H, F, [ctx, max(0, ctx - 1)], 16, dtype="f32")
    for b in range(2):
        y, k_new, v_new = _run(c, b)
        ty, tk, tv = _torch_layer(c, b)
        assert np.allclose(y, ty, rtol=1e-10, atol=1e-11)
        assert np.allclose(k_new, tk, rtol=1e-11, atol=1e-12) and np.allclose(v_new, tv, rtol=1e-12, atol=1e-13)
