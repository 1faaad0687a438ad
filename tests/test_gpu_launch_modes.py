"""GPU tests of how the step is launched rather than of what it computes: the prepared-call path that the
benchmark times, replay from a captured HIP graph, and the draft-head timing hook.

Each compares the library with itself (eager, freshly marshalled calls); the comparison with the oracle is in
test_gpu_parity.py.
"""
import math

import numpy as np
import pytest
import torch

import workloads
from gpu_harness import cached_inputs
from workloads.device import dev_f32, dev_i32, dev_i64, to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pkg():
    import paper_2412_00061_amd as m
    m.load_library()
    return m


class _Step:
    """Buffers and prepared calls of one step of a configuration, as bench.py sets them up."""

    def __init__(self, pkg, cfg_index, seed=0, variant="literal"):
        from paper_2412_00061_amd.binding import CTCSPEC_BF16, CTCSPEC_F32
        self.pkg = pkg
        cfg = self.cfg = workloads.get_config(cfg_index)
        x = self.x = cached_inputs(cfg_index, seed, variant)
        self.ctx = pkg.Context.for_config(cfg)
        B, T, k, N, H, dh = cfg.B, cfg.T, cfg.k, cfg.max_nodes, cfg.H, cfg.dh
        dt = CTCSPEC_BF16 if cfg.dtype == "bf16" else CTCSPEC_F32
        self.keep = [to_device(x.hidden, cfg.dtype), to_device(x.w, cfg.dtype), dev_f32(x.bias),
                     dev_i32(x.root_token)]
        d_hidden, d_w, d_bias, d_root = self.keep
        q, kt, vt, kc, vc = (to_device(a, cfg.dtype) for a in (x.q, x.k_tree, x.v_tree, x.k_cache, x.v_cache))
        d_off, d_len = dev_i64(x.kv_off), dev_i32(x.ctx_len)
        self.keep += [q, kt, vt, kc, vc, d_off, d_len]

        def i32(*shape):
            return torch.full(shape, -7, dtype=torch.int32, device="cuda")

        def f32(*shape):
            return torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")

        words = (N + 63) // 64
        o = self.out = dict(
            topk_id=i32(B, T, k), topk_logp=f32(B, T, k), lse=f32(B, T),
            n_cand=i32(B), cand_tokens=i32(B, cfg.beam, T), cand_len=i32(B, cfg.beam),
            cand_score=f32(B, cfg.beam), cand_leaf=i32(B, cfg.beam),
            n_nodes=i32(B), node_token=i32(B, N), node_parent=i32(B, N), node_depth=i32(B, N),
            anc_mask=torch.zeros((B, N, words), dtype=torch.int64, device="cuda"),
            attn=f32(B, H, N, dh),
            accept_len=i32(B), accept_nodes=i32(B, T + 1), accept_tokens=i32(B, T + 1), next_token=i32(B))
        self.targets = torch.full((B, N), cfg.V + 5, dtype=torch.int32, device="cuda")
        ctx, scale = self.ctx, 1.0 / math.sqrt(dh)
        self.calls = (
            pkg.prepared(ctx, "ctc_draft_topk", dt, d_hidden, d_w, d_bias, B, T, cfg.D, cfg.Vp1, k, o["topk_id"],
                         o["topk_logp"], o["lse"], None),
            pkg.prepared(ctx, "ctc_collapse_tree", o["topk_id"], o["topk_logp"], d_root, B, T, k, cfg.blank_id,
                         cfg.beam, N, o["n_cand"], o["cand_tokens"], o["cand_len"], o["cand_score"],
                         o["cand_leaf"], o["n_nodes"], o["node_token"], o["node_parent"], o["node_depth"],
                         o["anc_mask"]),
            pkg.prepared(ctx, "tree_verify_attn", dt, q, kc, vc, d_off, d_len, cfg.kv_cap, kt, vt, o["n_nodes"],
                         o["anc_mask"], B, H, dh, N, scale, o["attn"]),
            pkg.prepared(ctx, "accept_longest", o["n_nodes"], o["node_token"], o["node_parent"], o["node_depth"],
                         self.targets, B, T, N, o["accept_len"], o["accept_nodes"], o["accept_tokens"],
                         o["next_token"]),
        )

    def run(self):
        for c in self.calls:
            c()

    def snapshot(self):
        torch.cuda.synchronize()
        n = self.out["n_nodes"].cpu().numpy()
        snap = {}
        for name, t in self.out.items():
            a = t.cpu().numpy().copy()
            if name == "attn":  # rows of nodes that do not exist are not written
                for b in range(a.shape[0]):
                    a[b, :, n[b]:] = 0
            snap[name] = a
        return snap

    def scrub(self):
        for name, t in self.out.items():
            if t.dtype == torch.float32:
                t.fill_(float("nan"))
            else:
                t.fill_(-7 if name != "anc_mask" else 0)

    def plant_targets(self):
        """Make the acceptance walk follow the deepest path of the tree the step produced."""
        torch.cuda.synchronize()
        cfg = self.cfg
        n = self.out["n_nodes"].cpu().numpy()
        par, tok, dep = (self.out[k].cpu().numpy() for k in ("node_parent", "node_token", "node_depth"))
        tgt = np.full((cfg.B, cfg.max_nodes), cfg.V + 5, dtype=np.int32)
        for b in range(cfg.B):
            node = int(np.argmax(dep[b, :n[b]]))
            while node > 0:
                tgt[b, par[b, node]] = tok[b, node]
                node = par[b, node]
        self.targets.copy_(torch.from_numpy(tgt))


def _same(a, b):
    for name in a:
        assert np.array_equal(a[name], b[name], equal_nan=True), name


@pytest.mark.parametrize("cfg_index", [0, 2])
def test_prepared_calls_match_fresh_calls(pkg, cfg_index):
    st = _Step(pkg, cfg_index)
    st.run()
    st.plant_targets()
    st.run()
    got = st.snapshot()
    cfg, ctx = st.cfg, st.ctx
    d_hidden, d_w, d_bias, d_root, q, kt, vt, kc, vc, d_off, d_len = st.keep
    s12 = pkg.ctc_draft_topk(ctx, d_hidden, d_w, d_bias, cfg.k)
    s3 = pkg.ctc_collapse_tree(ctx, s12["topk_id"], s12["topk_logp"], d_root, cfg.blank_id, cfg.beam,
                               cfg.max_nodes)
    attn = pkg.tree_verify_attn(ctx, q, kc, vc, d_off, d_len, cfg.kv_cap, kt, vt, s3["n_nodes"], s3["anc_mask"],
                                1.0 / math.sqrt(cfg.dh))
    acc = pkg.accept_longest(ctx, s3["n_nodes"], s3["node_token"], s3["node_parent"], s3["node_depth"],
                             st.targets, cfg.T)
    torch.cuda.synchronize()
    for name in ("topk_id", "topk_logp", "lse"):
        assert np.array_equal(got[name], s12[name].cpu().numpy()), name
    for name in ("n_cand", "cand_tokens", "cand_len", "cand_score", "cand_leaf", "n_nodes", "node_token",
                 "node_parent", "node_depth", "anc_mask"):
        assert np.array_equal(got[name], s3[name].cpu().numpy()), name
    n = got["n_nodes"]
    a = attn.cpu().numpy()
    for b in range(cfg.B):
        assert np.array_equal(got["attn"][b, :, :n[b]], a[b, :, :n[b]])
    for name in ("accept_len", "accept_nodes", "accept_tokens", "next_token"):
        assert np.array_equal(got[name], acc[name].cpu().numpy()), name
    assert int(got["accept_len"].max()) >= 1  # the planted path was followed
    ctx.close()


@pytest.mark.parametrize("cfg_index", [0, 2])
def test_graph_replay_matches_eager(pkg, cfg_index):
    """The whole step captured into one HIP graph: every replay, with eager work and synchronisation in
    between, must reproduce the eager results bit for bit."""
    st = _Step(pkg, cfg_index)
    st.run()
    st.plant_targets()
    st.run()
    eager = st.snapshot()

    stream = torch.cuda.Stream()
    st.ctx.set_stream(stream)
    with torch.cuda.stream(stream):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            st.run()
    torch.cuda.synchronize()
    for rep in range(4):
        st.scrub()
        torch.cuda.synchronize()
        graph.replay()
        _same(eager, st.snapshot())
        # eager work of the program between the replays
        st.ctx.set_stream(torch.cuda.current_stream())
        st.scrub()
        st.run()
        _same(eager, st.snapshot())
        st.ctx.set_stream(stream)
    st.ctx.set_stream(torch.cuda.current_stream())
    st.ctx.close()


def test_draft_head_timing_hook(pkg):
    st = _Step(pkg, 2)
    ctx = st.ctx
    with pytest.raises(pkg.CtcspecError):
        ctx.draft_head_kernel_ms()  # profiling is off
    ctx.profile_draft_head(True)
    with pytest.raises(pkg.CtcspecError):
        ctx.draft_head_kernel_ms()  # nothing recorded yet
    st.calls[0]()
    ms = ctx.draft_head_kernel_ms()
    assert 0.005 < ms < 5.0  # 262 MB cannot be read in under 5 us; 5 ms would be 100 times too slow
    st.calls[0]()
    torch.cuda.synchronize()
    t = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t[0].record()
    st.calls[0]()
    t[1].record()
    torch.cuda.synchronize()
    assert ctx.draft_head_kernel_ms() <= t[0].elapsed_time(t[1]) + 0.02  # the kernel alone vs the whole call
    ctx.profile_draft_head(False)
    with pytest.raises(pkg.CtcspecError):
        ctx.draft_head_kernel_ms()
    ctx.close()


@pytest.mark.parametrize("cfg_index", [1, 2, 3, 4])
def test_attention_repeats_bit_identically(pkg, cfg_index):
    """Same inputs, same launch: the output must not depend on timing (a softmax reference that differed from
    run to run - an unreliable lane exchange - once showed up only here, far inside the parity tolerance)."""
    cfg = workloads.get_config(cfg_index)
    x = cached_inputs(cfg_index, 0, "literal")
    ctx = pkg.Context.for_config(cfg)
    q, kt, vt, kc, vc = (to_device(a, cfg.dtype) for a in (x.q, x.k_tree, x.v_tree, x.k_cache, x.v_cache))
    d_off, d_len = dev_i64(x.kv_off), dev_i32(x.ctx_len)
    N = cfg.max_nodes
    words = (N + 63) // 64
    mask = np.zeros((cfg.B, N, words), dtype=np.uint64)
    for i in range(N):  # a full binary tree: node i hangs under (i - 1) // 2
        a = i
        while True:
            mask[:, i, a >> 6] |= np.uint64(1) << np.uint64(a & 63)
            if a == 0:
                break
            a = (a - 1) // 2
    d_mask = torch.from_numpy(mask.view(np.int64)).cuda()
    n_nodes = torch.full((cfg.B,), N, dtype=torch.int32, device="cuda")
    outs = []
    for _ in range(4):
        o = pkg.tree_verify_attn(ctx, q, kc, vc, d_off, d_len, cfg.kv_cap, kt, vt, n_nodes, d_mask,
                                 1.0 / math.sqrt(cfg.dh))
        torch.cuda.synchronize()
        outs.append(o.cpu().numpy())
    for o in outs[1:]:
        assert np.array_equal(o, outs[0])
    ctx.close()


def whole_decode_step_graph_replay(pkg, capture_first):
    """Every call of a decode step in one HIP graph - the draft module's layer, the draft head, collapse/tree,
    the Eq. 5 values, verification attention, the base head, acceptance and the history update: replays,
    with eager work and synchronisation between them, must reproduce the eager results bit for bit (the
    history update writes the same rows each time: ctx_len is an input, the new length goes to its own buffer)."""
    from paper_2412_00061_amd.binding import CTCSPEC_BF16
    B, T, k, D, H, F, V, N, beam, cap = 1, 8, 4, 256, 2, 512, 400, 32, 32, 96
    dh = D // H
    c = workloads.make_draft_layer_case(21, B, T, D, H, F, [40], cap, dtype="bf16")
    rng = np.random.Generator(np.random.PCG64(22))
    rnd = lambda *s, scale=1.0: workloads.round_to_storage(rng.standard_normal(s, dtype=np.float32) * scale, "bf16")
    ctx = pkg.Context(max_batch=B, max_slots=T, max_topk=k, max_vocab_rows=V + 1, max_nodes=N, max_heads=H,
                      max_head_dim=dh)
    w = c.weights
    lw = pkg.layer_weights(to_device(w["ln1"], "bf16"), to_device(np.concatenate([w["wq"], w["wk"], w["wv"]]), "bf16"),
                           to_device(w["wo"], "bf16"), to_device(w["ln2"], "bf16"),
                           to_device(np.concatenate([w["wg"], w["wu"]]), "bf16"), to_device(w["wd"], "bf16"))
    x_in, pos0 = to_device(c.x, "bf16"), dev_i32(c.pos0)
    kc_draft, vc_draft = to_device(c.k_cache, "bf16"), to_device(c.v_cache, "bf16")
    d_off, d_len = dev_i64(c.kv_off), dev_i32(c.ctx_len)
    w_draft, w_base = to_device(rnd(V + 1, D, scale=0.05), "bf16"), to_device(rnd(V, D, scale=0.05), "bf16")
    q, kt, vt = (to_device(rnd(B, H, N, dh), "bf16") for _ in range(3))
    kc, vc = to_device(np.nan_to_num(c.k_cache), "bf16"), to_device(np.nan_to_num(c.v_cache), "bf16")
    node_hidden = to_device(rnd(B, N, D), "bf16")
    root = dev_i32(np.array([7], dtype=np.int32))

    def i32(*shape):
        return torch.full(shape, -7, dtype=torch.int32, device="cuda")

    def f32(*shape):
        return torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")

    ws = torch.empty(pkg.draft_layer_workspace_bytes(B, T, D, H, F), dtype=torch.uint8, device="cuda")
    bf = lambda *shape: torch.zeros(shape, dtype=torch.bfloat16, device="cuda")
    o = dict(slot=bf(B, T, D), k_new=bf(B, H, T, dh), v_new=bf(B, H, T, dh),
             topk_id=i32(B, T, k), topk_logp=f32(B, T, k), lse=f32(B, T), logits=f32(B, T, V + 1),
             n_cand=i32(B), cand_tokens=i32(B, beam, T), cand_len=i32(B, beam), cand_score=f32(B, beam),
             cand_leaf=i32(B, beam), n_nodes=i32(B), node_token=i32(B, N), node_parent=i32(B, N),
             node_depth=i32(B, N), anc_mask=torch.zeros((B, N, 1), dtype=torch.int64, device="cuda"),
             sum=f32(B, beam), rank=i32(B, beam), attn=f32(B, H, N, dh), target=i32(B, N),
             accept_len=i32(B), accept_nodes=i32(B, T + 1), accept_tokens=i32(B, T + 1), next_token=i32(B),
             new_len=i32(B))
    P = pkg.prepared
    calls = (
        P(ctx, "draft_layer_forward", CTCSPEC_BF16, x_in, lw, pos0, kc_draft, vc_draft, d_off, d_len, cap, B, T, D, H, F,
          c.eps, c.theta, ws, ws.numel(), None, o["k_new"], o["v_new"], o["slot"], None),
        P(ctx, "ctc_draft_topk", CTCSPEC_BF16, o["slot"], w_draft, None, B, T, D, V + 1, k, o["topk_id"],
          o["topk_logp"], o["lse"], o["logits"]),
        P(ctx, "ctc_collapse_tree", o["topk_id"], o["topk_logp"], root, B, T, k, V, beam, N, o["n_cand"],
          o["cand_tokens"], o["cand_len"], o["cand_score"], o["cand_leaf"], o["n_nodes"], o["node_token"],
          o["node_parent"], o["node_depth"], o["anc_mask"]),
        P(ctx, "ctc_sum_score", o["logits"], o["lse"], o["cand_tokens"], o["cand_len"], o["n_cand"], B, T, V + 1, V,
          beam, o["sum"], o["rank"]),
        P(ctx, "tree_verify_attn", CTCSPEC_BF16, q, kc, vc, d_off, d_len, cap, kt, vt, o["n_nodes"], o["anc_mask"],
          B, H, dh, N, 1.0 / math.sqrt(dh), o["attn"]),
        P(ctx, "verify_head_argmax", CTCSPEC_BF16, node_hidden, w_base, o["n_nodes"], B, N, D, V, o["target"], None),
        P(ctx, "accept_longest", o["n_nodes"], o["node_token"], o["node_parent"], o["node_depth"], o["target"], B, T,
          N, o["accept_len"], o["accept_nodes"], o["accept_tokens"], o["next_token"]),
        P(ctx, "kv_commit", CTCSPEC_BF16, kt, vt, o["accept_len"], o["accept_nodes"], T, d_off, d_len, cap, B, H, dh,
          N, kc, vc, o["new_len"]),
    )

    def run():
        for call in calls:
            call()

    def snapshot():
        torch.cuda.synchronize()
        n = int(o["n_nodes"][0])
        snap = {}
        for name, t in o.items():
            a = t.float().cpu().numpy().copy() if t.dtype == torch.bfloat16 else t.cpu().numpy().copy()
            if name == "attn":
                a[:, :, n:] = 0
            snap[name] = a
        snap["kc"], snap["vc"] = kc.float().cpu().numpy().copy(), vc.float().cpu().numpy().copy()
        return snap

    def scrub():
        for name, t in o.items():
            if t.dtype == torch.float32:
                t.fill_(float("nan"))
            elif t.dtype == torch.bfloat16:
                t.zero_()
            else:
                t.fill_(-7 if name != "anc_mask" else 0)

    stream = torch.cuda.Stream()
    if capture_first:
        # the stage calls' very first use in this process is the one the capture records: nothing they do may need
        # an eager call first (function attributes and code loading belong to ctcspec_create)
        ctx.set_stream(stream)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            run()
        torch.cuda.synchronize()
        graph.replay()
        first = snapshot()
        ctx.set_stream(torch.cuda.current_stream())
        scrub()
        run()
        eager = snapshot()
        _same(eager, first)
        ctx.set_stream(stream)
    else:
        run()
        eager = snapshot()
        ctx.set_stream(stream)
        with torch.cuda.stream(stream):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                run()
        torch.cuda.synchronize()
    assert int(eager["n_nodes"][0]) > 1 and int(eager["new_len"][0]) == 40 + int(eager["accept_len"][0]) + 1
    for rep in range(3):
        scrub()
        torch.cuda.synchronize()
        graph.replay()
        _same(eager, snapshot())
        junk = torch.randn(1 << 16, device="cuda").sum()  # eager work between the replays
        torch.cuda.synchronize()
        assert math.isfinite(float(junk))
    ctx.set_stream(torch.cuda.current_stream())
    ctx.close()


def test_whole_decode_step_graph_replay(pkg):
    whole_decode_step_graph_replay(pkg, capture_first=False)


def test_first_calls_after_create_are_capturable():
    """A fresh process whose first stage calls are recorded by a stream capture (see capture_first_call.py): no call
    may rely on an eager call having gone before it."""
    import os
    import subprocess
    import sys
    here = os.path.dirname(os.path.abspath(__file__))
    res = subprocess.run([sys.executable, os.path.join(here, "capture_first_call.py")], capture_output=True, text=True,
                         timeout=300)
    assert res.returncode == 0 and "capture-first ok" in res.stdout, res.stdout[-2000:] + res.stderr[-4000:]


def test_loss_and_sampled_draw_graph_replay(pkg):
    """ctc_loss (with its gradient) and the sampled draw followed by the acceptance walk, captured in one HIP graph:
    replays, with eager work and synchronisation between them, reproduce the eager results bit for bit."""
    rng = np.random.Generator(np.random.PCG64(31))
    B, T, C, Lmax = 3, 12, 301, 6
    logits = dev_f32(rng.standard_normal((B, T, C), dtype=np.float32) * 2)
    labels = dev_i32(rng.integers(0, C - 1, size=(B, Lmax)).astype(np.int32))
    label_len = dev_i32(np.array([6, 0, 3], dtype=np.int32))
    frame_len = dev_i32(np.array([12, 5, 9], dtype=np.int32))
    N, V = 6, 301
    node_token = dev_i32(np.array([[9, 4, 5, 6, 7, 8]], dtype=np.int32))
    node_parent = dev_i32(np.array([[-1, 0, 0, 1, 1, 3]], dtype=np.int32))
    node_depth = dev_i32(np.array([[0, 1, 1, 2, 2, 3]], dtype=np.int32))
    n_nodes = dev_i32(np.array([N], dtype=np.int32))
    z = rng.standard_normal((1, N, V), dtype=np.float32)
    z[0, 0, 4] += 9.0
    z[0, 1, 6] += 9.0
    uniforms = dev_f32(rng.random((1, N), dtype=np.float32))
    z = dev_f32(z)
    ctx = pkg.Context(max_batch=B, max_slots=8, max_topk=4, max_vocab_rows=C, max_nodes=8, max_heads=1, max_head_dim=8)
    ws = torch.empty(pkg.ctc_loss_workspace_bytes(B, T, Lmax), dtype=torch.uint8, device="cuda")
    o = dict(loss=torch.full((B,), float("nan"), device="cuda"), grad=torch.full((B, T, C), float("nan"), device="cuda"),
             drawn=torch.full((1, N), -7, dtype=torch.int32, device="cuda"),
             accept_len=torch.full((1,), -7, dtype=torch.int32, device="cuda"),
             accept_nodes=torch.full((1, 5), -7, dtype=torch.int32, device="cuda"),
             accept_tokens=torch.full((1, 5), -7, dtype=torch.int32, device="cuda"),
             next_token=torch.full((1,), -7, dtype=torch.int32, device="cuda"))
    P = pkg.prepared
    calls = (
        P(ctx, "ctc_loss", logits, labels, label_len, frame_len, B, T, C, Lmax, C - 1, ws, ws.numel(), o["loss"], o["grad"]),
        P(ctx, "verify_sample_tokens", z, n_nodes, uniforms, 0.9, 1, N, V, o["drawn"]),
        P(ctx, "accept_longest", n_nodes, node_token, node_parent, node_depth, o["drawn"], 1, 4, N, o["accept_len"],
          o["accept_nodes"], o["accept_tokens"], o["next_token"]),
    )

    def run():
        for call in calls:
            call()

    def snapshot():
        torch.cuda.synchronize()
        return {name: t.cpu().numpy().copy() for name, t in o.items()}

    run()
    eager = snapshot()
    assert np.isfinite(eager["loss"]).all() and int(eager["accept_len"][0]) >= 1
    stream = torch.cuda.Stream()
    ctx.set_stream(stream)
    with torch.cuda.stream(stream):
        run()
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            run()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in o.values():
            t.fill_(float("nan") if t.dtype == torch.float32 else -7)
        torch.cuda.synchronize()
        graph.replay()
        _same(eager, snapshot())
        junk = torch.randn(1 << 16, device="cuda").sum()
        torch.cuda.synchronize()
        assert math.isfinite(float(junk))
    ctx.set_stream(torch.cuda.current_stream())
    ctx.close()


# ------------------------------------------------------------------------------ deferred merge of the draft head
def _draft_and_tree(pkg, ctx, st, k, beam, N):
    cfg = st.cfg
    d_hidden, d_w, d_bias, d_root = st.keep[:4]
    s12 = pkg.ctc_draft_topk(ctx, d_hidden, d_w, d_bias, k)
    s3 = pkg.ctc_collapse_tree(ctx, s12["topk_id"], s12["topk_logp"], d_root, cfg.blank_id, beam, N)
    torch.cuda.synchronize()
    return {**{n: t.cpu().numpy() for n, t in s12.items()}, **{n: t.cpu().numpy() for n, t in s3.items()}}


@pytest.mark.parametrize("cfg_index,variant", [(0, "ar1"), (2, "literal"), (2, "structured"), (4, "structured")])
def test_deferred_merge_gives_the_same_bits(pkg, cfg_index, variant):
    """ctc_draft_topk with its merge left to ctc_collapse_tree's kernel: every output of both calls must equal the
    two-kernel path bit for bit (the merge is the same code in both places)."""
    st = _Step(pkg, cfg_index, variant=variant)
    cfg, ctx = st.cfg, st.ctx
    plain = _draft_and_tree(pkg, ctx, st, cfg.k, cfg.beam, cfg.max_nodes)
    ctx.defer_topk_merge(True)
    fused = _draft_and_tree(pkg, ctx, st, cfg.k, cfg.beam, cfg.max_nodes)
    again = _draft_and_tree(pkg, ctx, st, cfg.k, cfg.beam, cfg.max_nodes)
    ctx.defer_topk_merge(False)
    for name in plain:
        assert np.array_equal(plain[name].view(np.uint8), fused[name].view(np.uint8)), name
        assert np.array_equal(plain[name].view(np.uint8), again[name].view(np.uint8)), name
    ctx.close()


def test_deferred_merge_is_settled_by_whatever_comes_next(pkg):
    """The owed lists appear whatever the next call is: ctcspec_flush, another stage call, a collapse call on other
    buffers or with a list length the built-in merge does not cover, a second draft call, a stream change."""
    st = _Step(pkg, 1)
    cfg, ctx = st.cfg, st.ctx
    d_hidden, d_w, d_bias, d_root = st.keep[:4]
    want = pkg.ctc_draft_topk(ctx, d_hidden, d_w, d_bias, cfg.k)
    torch.cuda.synchronize()
    ctx.defer_topk_merge(True)

    def owed(k=cfg.k):
        out = {"topk_id": torch.full((cfg.B, cfg.T, k), -7, dtype=torch.int32, device="cuda"),
               "topk_logp": torch.full((cfg.B, cfg.T, k), float("nan"), device="cuda"),
               "lse": torch.full((cfg.B, cfg.T), float("nan"), device="cuda")}
        return pkg.ctc_draft_topk(ctx, d_hidden, d_w, d_bias, k, out=out)

    def settled(got, ref=want):
        torch.cuda.synchronize()
        for name in ref:
            assert torch.equal(got[name].view(torch.int32), ref[name].view(torch.int32)), name

    got = owed()
    ctx.flush()
    settled(got)
    got = owed()
    pkg.accept_longest(ctx, st.out["n_nodes"].fill_(1), st.out["node_token"], st.out["node_parent"], st.out["node_depth"],
                       st.targets, cfg.T)
    settled(got)
    got = owed()
    ids2, lp2 = want["topk_id"].clone(), want["topk_logp"].clone()  # a collapse call on other buffers
    pkg.ctc_collapse_tree(ctx, ids2, lp2, d_root, cfg.blank_id, cfg.beam, cfg.max_nodes)
    settled(got)
    got = owed()
    pkg.ctc_raw_tree(ctx, got["topk_id"], got["topk_logp"], d_root, cfg.blank_id, cfg.beam, cfg.max_nodes)
    settled(got)
    # lists of five keys: the collapse kernel's built-in merge stops at four, so it launches the merge kernel first
    rng = np.random.Generator(np.random.PCG64(5))
    h5 = to_device(workloads.round_to_storage(rng.standard_normal((1, 4, 512), dtype=np.float32), "bf16"), "bf16")
    w5 = to_device(workloads.round_to_storage(rng.standard_normal((300, 512), dtype=np.float32) * 0.05, "bf16"), "bf16")
    ctx5 = pkg.Context(max_batch=1, max_slots=4, max_topk=5, max_vocab_rows=300, max_nodes=32, max_heads=1,
                       max_head_dim=16)
    want5 = pkg.ctc_draft_topk(ctx5, h5, w5, None, 5)
    tree5 = pkg.ctc_collapse_tree(ctx5, want5["topk_id"], want5["topk_logp"], d_root, 299, 16, 32)
    ctx5.defer_topk_merge(True)
    got5 = pkg.ctc_draft_topk(ctx5, h5, w5, None, 5)
    got_tree5 = pkg.ctc_collapse_tree(ctx5, got5["topk_id"], got5["topk_logp"], d_root, 299, 16, 32)
    settled(got5, want5)
    for name in tree5:
        assert torch.equal(tree5[name], got_tree5[name]), name
    ctx5.close()
    first = owed()
    second = owed()  # the second call's partials overwrite the first's: the first must have been merged before
    ctx.flush()
    settled(first)
    settled(second)
    got = owed()
    other = torch.cuda.Stream()
    ctx.set_stream(other)  # settles on the stream the partials were produced on
    other.synchronize()
    settled(got)
    ctx.set_stream(torch.cuda.current_stream())
    ctx.defer_topk_merge(False)
    ctx.close()


def test_deferred_merge_graph_replay(pkg):
    """The step with the deferred merge, captured and replayed: the same results as eager calls without it."""
    st = _Step(pkg, 2)
    st.run()
    st.plant_targets()
    st.run()
    eager = st.snapshot()
    stream = torch.cuda.Stream()
    st.ctx.defer_topk_merge(True)
    st.ctx.set_stream(stream)
    with torch.cuda.stream(stream):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            st.run()
    torch.cuda.synchronize()
    for rep in range(3):
        st.scrub()
        torch.cuda.synchronize()
        graph.replay()
        _same(eager, st.snapshot())
    st.ctx.set_stream(torch.cuda.current_stream())
    st.ctx.defer_topk_merge(False)
    st.ctx.close()
