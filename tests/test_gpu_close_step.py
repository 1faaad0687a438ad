"""GPU parity of the two calls that close the step: verify_head_argmax and kv_commit, against the oracle.

Logits within 2e-3 (relative, RMS floor; bf16 inputs, fp32 accumulation); the greedy token is decided on the
kernel's own fp32 logits and must then match bit for bit, ties to the smaller id; cache rows and lengths are
copies and must match bit for bit.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_harness import rel_err_rms_floor
from workloads.device import dev_i32, dev_i64, to_device

pytestmark = pytest.mark.gpu
TOL = 2e-3


@pytest.fixture(scope="module")
def pkg():
    import paper_2412_00061_amd as m
    m.load_library()
    return m


def _check_head(pkg, B, N, D, V, dtype, n_nodes, seed, dup_rows=()):
    rng = np.random.Generator(np.random.PCG64(seed))
    hidden = workloads.round_to_storage(rng.standard_normal((B, N, D), dtype=np.float32), dtype)
    w = workloads.round_to_storage(rng.standard_normal((V, D), dtype=np.float32) * 0.05, dtype)
    for a, b in dup_rows:  # exactly equal logits for two ids
        w[a] = w[b]
    ctx = pkg.Context(max_batch=B, max_slots=8, max_topk=4, max_vocab_rows=V, max_nodes=N, max_heads=1,
                      max_head_dim=16)
    dh, dw, dn = to_device(hidden, dtype), to_device(w, dtype), dev_i32(np.asarray(n_nodes, dtype=np.int32))
    res = pkg.verify_head_argmax(ctx, dh, dw, dn, want_logits=True)
    fast = pkg.verify_head_argmax(ctx, dh, dw, dn)
    torch.cuda.synchronize()
    z_gpu = res["logits"].cpu().numpy()
    got = res["target_argmax"].cpu().numpy()
    for b in range(B):
        z_ref, _ = oracle.verifier_head_argmax(hidden[b], w, int(n_nodes[b]))
        n = int(n_nodes[b])
        assert rel_err_rms_floor(z_gpu[b, :n], z_ref[:n]) <= TOL
        assert np.array_equal(got[b], oracle.argmax_rows(z_gpu[b], n))
    assert torch.equal(res["target_argmax"], fast["target_argmax"])
    ctx.close()
    return got, z_gpu


@pytest.mark.parametrize("cfg_index", [2, 3, 4])
def test_verify_head_full_size(pkg, cfg_index):
    cfg = workloads.get_config(cfg_index)
    rng = np.random.Generator(np.random.PCG64(cfg_index))
    n_nodes = rng.integers(1, cfg.max_nodes + 1, size=cfg.B)
    n_nodes[0] = cfg.max_nodes
    _check_head(pkg, cfg.B, cfg.max_nodes, cfg.D, cfg.V, cfg.dtype, n_nodes, seed=cfg_index)


@pytest.mark.parametrize("B,N,D,V,dtype", [
    (1, 128, 1024, 1000, "bf16"),   # MFMA kernel, ragged last row block
    (2, 100, 2048, 129, "bf16"),    # 200 columns: two column blocks, the second ragged; vocabulary barely past a block
    (3, 100, 1024, 1100, "bf16"),   # 300 columns: three column blocks over five row blocks of 256 (fewer than the 8 XCDs), ragged last one
    (5, 128, 512, 2200, "bf16"),    # five full column blocks, nine row blocks of 256: one XCD sees two row groups
    (3, 100, 512, 5000, "bf16"),    # three column blocks over twenty row blocks of 256: several row groups per XCD
    (1, 5, 1024, 77, "bf16"),       # fewer rows than a block, few columns
    (3, 16, 512, 300, "bf16"),      # hidden size the MFMA kernel does not take: generic kernel
    (2, 9, 48, 11, "f32"),
    (1, 1, 8, 1, "f32"),            # a single token in the vocabulary
])
def test_verify_head_shapes(pkg, B, N, D, V, dtype):
    rng = np.random.Generator(np.random.PCG64(B * 100 + N))
    n_nodes = rng.integers(1, N + 1, size=B)
    _check_head(pkg, B, N, D, V, dtype, n_nodes, seed=D + V)


def test_verify_head_ties_go_to_the_smaller_id(pkg):
    # rows 7, 300 and 650 of the head are identical and made dominant: every node's greedy token is 7
    rng = np.random.Generator(np.random.PCG64(5))
    B, N, D, V = 1, 40, 1024, 700
    hidden = workloads.round_to_storage(np.abs(rng.standard_normal((B, N, D), dtype=np.float32)), "bf16")
    w = workloads.round_to_storage(rng.standard_normal((V, D), dtype=np.float32) * 0.02, "bf16")
    w[650] = w[300] = w[7] = workloads.round_to_storage(np.full(D, 0.5, dtype=np.float32), "bf16")
    ctx = pkg.Context(max_batch=B, max_slots=8, max_topk=4, max_vocab_rows=V, max_nodes=N, max_heads=1, max_head_dim=16)
    res = pkg.verify_head_argmax(ctx, to_device(hidden, "bf16"), to_device(w, "bf16"), dev_i32(np.array([N], np.int32)),
                                 want_logits=True)
    torch.cuda.synchronize()
    z = res["logits"].cpu().numpy()[0]
    assert np.array_equal(z[:, 7], z[:, 300]) and np.array_equal(z[:, 7], z[:, 650])
    assert (res["target_argmax"].cpu().numpy()[0] == 7).all()
    ctx.close()


@pytest.mark.parametrize("cfg_index,seed", [(0, 0), (2, 1), (4, 2)])
def test_kv_commit_matches_oracle(pkg, cfg_index, seed):
    cfg = workloads.get_config(cfg_index)
    x = workloads.make_inputs(cfg, seed, "literal")
    rng = np.random.Generator(np.random.PCG64(seed))
    B, T, N, H, dh = cfg.B, cfg.T, cfg.max_nodes, cfg.H, cfg.dh
    ctx_len = np.array(x.ctx_len, dtype=np.int32).copy()
    ctx_len[0] = cfg.kv_cap - 2            # the first sequence runs out of room: saturation
    accept_len = rng.integers(0, T + 1, size=B).astype(np.int32)
    accept_len[0] = min(T, 4)
    accept_nodes = np.full((B, T + 1), -1, dtype=np.int32)
    for b in range(B):
        accept_nodes[b, 0] = 0
        accept_nodes[b, 1:accept_len[b] + 1] = rng.choice(np.arange(1, N), size=accept_len[b], replace=False)
    ctx = pkg.Context.for_config(cfg)
    d_kc, d_vc = to_device(x.k_cache, cfg.dtype), to_device(x.v_cache, cfg.dtype)
    d_kt, d_vt = to_device(x.k_tree, cfg.dtype), to_device(x.v_tree, cfg.dtype)
    new_len = torch.full((B,), -5, dtype=torch.int32, device="cuda")
    kc0, vc0 = d_kc.clone(), d_vc.clone()
    pkg.kv_commit(ctx, d_kt, d_vt, dev_i32(accept_len), dev_i32(accept_nodes), dev_i64(x.kv_off), dev_i32(ctx_len),
                  cfg.kv_cap, d_kc, d_vc, ctx_len_out=new_len)
    torch.cuda.synchronize()

    def bits(t):  # compare raw bits: rows beyond the context hold NaN on purpose
        return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).cpu().numpy().reshape(-1)

    got_k, got_v, old_k, old_v = bits(d_kc), bits(d_vc), bits(kc0), bits(vc0)
    kt, vt = bits(d_kt).reshape(B, H, N, dh), bits(d_vt).reshape(B, H, N, dh)
    for b in range(B):
        off = int(x.kv_off[b])
        sl = slice(off, off + H * cfg.kv_cap * dh)
        want_k, want_v, want_len = oracle.kv_commit(old_k[sl].reshape(H, cfg.kv_cap, dh), old_v[sl].reshape(H, cfg.kv_cap, dh),
                                                    int(ctx_len[b]), kt[b], vt[b], int(accept_len[b]), accept_nodes[b])
        assert np.array_equal(got_k[sl].reshape(H, cfg.kv_cap, dh), want_k)
        assert np.array_equal(got_v[sl].reshape(H, cfg.kv_cap, dh), want_v)
        assert int(new_len[b]) == want_len
    assert int(new_len[0]) == cfg.kv_cap
    # without ctx_len_out nothing but the caches is touched; aliasing the length buffer is refused
    d_len = dev_i32(ctx_len)
    pkg.kv_commit(ctx, d_kt, d_vt, dev_i32(accept_len), dev_i32(accept_nodes), dev_i64(x.kv_off), d_len, cfg.kv_cap,
                  d_kc, d_vc)
    with pytest.raises(pkg.CtcspecError, match="ctx_len_out"):
        pkg.kv_commit(ctx, d_kt, d_vt, dev_i32(accept_len), dev_i32(accept_nodes), dev_i64(x.kv_off), d_len,
                      cfg.kv_cap, d_kc, d_vc, ctx_len_out=d_len)
    torch.cuda.synchronize()
    assert np.array_equal(d_len.cpu().numpy(), ctx_len)
    ctx.close()


def test_closed_step_feeds_the_next_step(pkg):
    """Tiny config end to end: draft, tree, attention, verifier head on a projection of the attention output,
    acceptance, history update - then attention of the NEXT step over the grown cache equals the oracle's on
    the oracle-updated cache."""
    cfg = workloads.get_config(0)
    x = workloads.make_inputs(cfg, 0, "ar1")
    ctx = pkg.Context.for_config(cfg)
    B, T, N, H, dh = cfg.B, cfg.T, cfg.max_nodes, cfg.H, cfg.dh
    scale = 1.0 / math.sqrt(dh)
    dt = cfg.dtype
    d_q, d_kt, d_vt = (to_device(a, dt) for a in (x.q, x.k_tree, x.v_tree))
    d_kc, d_vc = to_device(x.k_cache, dt), to_device(x.v_cache, dt)
    # room to grow: the tiny config's cache is exactly full, so the step starts two rows short of it
    ctx_len = np.maximum(np.array(x.ctx_len, dtype=np.int32) - (T + 1), 1)
    d_len, d_off = dev_i32(ctx_len), dev_i64(x.kv_off)
    s12 = pkg.ctc_draft_topk(ctx, to_device(x.hidden, dt), to_device(x.w, dt), torch.from_numpy(x.bias).cuda(), cfg.k)
    s3 = pkg.ctc_collapse_tree(ctx, s12["topk_id"], s12["topk_logp"], dev_i32(x.root_token), cfg.blank_id, cfg.beam, N)
    out = pkg.tree_verify_attn(ctx, d_q, d_kc, d_vc, d_off, d_len, cfg.kv_cap, d_kt, d_vt, s3["n_nodes"],
                               s3["anc_mask"], scale)
    # the node's "last hidden state": the heads of its attention output, concatenated (the rest of the base
    # model is out of scope); the head is the seeded projection of the workload
    node_hidden = out.permute(0, 2, 1, 3).reshape(B, N, H * dh).contiguous()
    vh = pkg.verify_head_argmax(ctx, node_hidden, to_device(x.proj, dt), s3["n_nodes"], want_logits=True)
    acc = pkg.accept_longest(ctx, s3["n_nodes"], s3["node_token"], s3["node_parent"], s3["node_depth"],
                             vh["target_argmax"], T)
    new_len = torch.zeros((B,), dtype=torch.int32, device="cuda")
    kc_before, vc_before = d_kc.cpu().numpy().copy(), d_vc.cpu().numpy().copy()
    pkg.kv_commit(ctx, d_kt, d_vt, acc["accept_len"], acc["accept_nodes"], d_off, d_len, cfg.kv_cap, d_kc, d_vc,
                  ctx_len_out=new_len)
    torch.cuda.synchronize()
    n = int(s3["n_nodes"][0])
    # verifier head on the kernel's own attention output
    z_ref, _ = oracle.verifier_head_argmax(node_hidden[0].cpu().numpy(), x.proj, n)
    assert rel_err_rms_floor(vh["logits"][0, :n].cpu().numpy(), z_ref[:n]) <= TOL
    target = vh["target_argmax"][0].cpu().numpy()
    assert np.array_equal(target, oracle.argmax_rows(vh["logits"][0].cpu().numpy(), n))
    # acceptance and history update chained on it
    length, nodes, toks, nxt = oracle.accept_longest(s3["node_token"][0].cpu().numpy(), s3["node_parent"][0].cpu().numpy(),
                                                     n, target, T)
    assert int(acc["accept_len"][0]) == length and int(acc["next_token"][0]) == nxt
    want_k, want_v, want_len = oracle.kv_commit(kc_before.reshape(H, cfg.kv_cap, dh), vc_before.reshape(H, cfg.kv_cap, dh),
                                                int(ctx_len[0]), x.k_tree[0], x.v_tree[0], length, nodes)
    assert int(new_len[0]) == want_len == int(ctx_len[0]) + length + 1
    assert np.array_equal(d_kc.cpu().numpy().reshape(H, cfg.kv_cap, dh), want_k)
    # the next step's attention sees the grown history
    out2 = pkg.tree_verify_attn(ctx, d_q, d_kc, d_vc, d_off, new_len, cfg.kv_cap, d_kt, d_vt, s3["n_nodes"],
                                s3["anc_mask"], scale)
    torch.cuda.synchronize()
    mask = np.zeros((N, N), dtype=bool)
    words = s3["anc_mask"][0].cpu().numpy().view(np.uint64)
    for i in range(n):
        for j in range(n):
            mask[i, j] = (int(words[i, j >> 6]) >> (j & 63)) & 1
    ref2 = oracle.tree_attention(x.q[0], want_k, want_v, want_len, x.k_tree[0], x.v_tree[0], n, mask, scale)
    assert rel_err_rms_floor(out2[0, :, :n].cpu().numpy(), ref2) <= TOL
    ctx.close()
