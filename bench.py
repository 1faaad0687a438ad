#!/usr/bin/env python3
"""Benchmark of one draft+verify step of CTC-drafted speculative decoding on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 7b_ctx2048] [--no-cpu-baseline]

A step is the whole hot path on one batch of seeded synthetic input that is already resident in HBM:
ctc_draft_topk -> ctc_collapse_tree -> tree_verify_attn (one attention layer) -> accept_longest, issued
back to back on one stream with no host synchronisation in between.  W untimed warm-up steps, then
exactly K timed steps between two device synchronisations.  To keep the 256 MB Infinity Cache from
serving the streams, the head weights rotate over several identical copies and the KV cache / Q / tree
K,V over many buffer sets, so every step reads memory that is not cached.

Prints ONE JSON line.  `value` is verified tokens per second (tree nodes pushed through verification
per second of step time); `roofline` describes the dominant kernel (the draft head, HBM-bound);
`cpu_baseline` is the float64 oracle timed on this machine's host cores on a bounded sample.
"""
import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", default="7b_ctx2048")
    ap.add_argument("--variant", default="literal", choices=["literal", "ar1", "structured"])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--w-copies", type=int, default=6)
    ap.add_argument("--kv-sets", type=int, default=32)
    ap.add_argument("--graph", action="store_true", help="replay the steps from a captured HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--deferred-merge", action="store_true",
                    help="leave the merge of the draft head's partial results to the collapse/tree kernel's prologue "
                         "(ctcspec_defer_topk_merge) instead of launching the merge kernel right behind the head")
    ap.add_argument("--attn-layers", type=int, default=-1,
                    help="layers of the full-depth variant line (attention called once per layer on its own "
                         "K/V/Q buffers); default: the layer count of the config (32 at 7B, 40 at 13B); 0: skip")
    ap.add_argument("--full-depth-steps", type=int, default=24)
    ap.add_argument("--no-closed-step", action="store_true")
    ap.add_argument("--no-draft-layer", action="store_true")
    ap.add_argument("--no-sum-score", action="store_true")
    ap.add_argument("--no-literal-layout", action="store_true")
    ap.add_argument("--no-ctc-loss", action="store_true")
    ap.add_argument("--no-sampled-acceptance", action="store_true")
    ap.add_argument("--ctc-loss-positions", type=int, default=4096,
                    help="training positions of the ctc_loss line, each with T frames over V+1 symbols")
    ap.add_argument("--draft-layer-ffn", type=int, default=0,
                    help="feed-forward width of the draft module's layer (0: the base family's, 43/16 of D)")
    ap.add_argument("--cpu-steps", type=int, default=12, help="oracle steps timed with all BLAS threads")
    ap.add_argument("--cpu-steps-one-thread", type=int, default=4, help="oracle steps timed with one BLAS thread")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run ten 256 MiB device copies (known traffic, for scaling rocprofv3 HBM counters)")
    return ap.parse_args()


def algorithmic_bytes(cfg, ctx_len, n_nodes):
    """Bytes one step must move by the method's own definition (weights and KV read once, small
    tensors once).  Returns (draft_head_bytes, attention_bytes, total)."""
    es = 2 if cfg.dtype == "bf16" else 4
    head = cfg.Vp1 * cfg.D * es + cfg.B * cfg.T * cfg.D * es + cfg.Vp1 * 4 + cfg.B * cfg.T * (2 * cfg.k + 1) * 4
    kv = int(sum(2 * int(L) * cfg.H * cfg.dh * es for L in ctx_len))
    qkv_tree = int(sum(3 * int(n) * cfg.H * cfg.dh * es for n in n_nodes))
    out = int(sum(int(n) * cfg.H * cfg.dh * 4 for n in n_nodes))
    small = cfg.B * (cfg.max_nodes * (16 + 8 * ((cfg.max_nodes + 63) // 64)) + cfg.beam * (cfg.T + 3) * 4)
    attn = kv + qkv_tree + out
    return head, attn, head + attn + small


def read_traffic_summary():
    """HBM bytes per draft-head launch from the committed rocprofv3 counter summary, or None."""
    path = os.path.join(ROOT, "profiles", "ctc_draft_topk_7b_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1].split()[0])
    except OSError:
        pass
    return None


def read_kernel_trace_us():
    """Average duration of the draft-head kernel in the committed rocprofv3 kernel trace (us), or None."""
    path = os.path.join(ROOT, "profiles", "step_7b_ctx2048_kernel_trace.txt")
    try:
        for line in open(path):
            if line.startswith("lmhead_bf16_mfma_kernel"):
                return float(line.split()[2])
    except (OSError, ValueError, IndexError):
        pass
    return None


def cpu_baseline(cfg, x, n_steps, n_steps_one_thread):
    """Time the float64 oracle, as it stands, on this host: n_steps whole steps of the same workload with all the cores
    its BLAS takes, then n_steps_one_thread with the BLAS held to one thread; per stage and in total."""
    import oracle
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threadpool_limits = None
        threads = os.cpu_count() or 1
    scale = 1.0 / math.sqrt(cfg.dh)
    stages = ("ctc_draft_topk", "ctc_collapse_tree", "tree_verify_attn", "accept_longest")

    def one_step():
        t = [time.perf_counter()]
        d = oracle.draft_topk(x.hidden, x.w, x.bias, cfg.k)
        t.append(time.perf_counter())
        trees = [oracle.collapse_tree(d["topk_id"][b], d["topk_logp"][b].astype(np.float32), int(x.root_token[b]),
                                      cfg.blank_id, cfg.beam, cfg.max_nodes) for b in range(cfg.B)]
        t.append(time.perf_counter())
        for b, tree in enumerate(trees):
            o = oracle.tree_attention(x.q[b], x.k_cache[b], x.v_cache[b], int(x.ctx_len[b]), x.k_tree[b], x.v_tree[b],
                                      tree["n_nodes"], tree["mask"], scale)
            del o
        t.append(time.perf_counter())
        for tree in trees:
            n = tree["n_nodes"]
            oracle.accept_longest(tree["node_token"], tree["node_parent"], n, np.full(n, -1, dtype=np.int32), cfg.T)
        t.append(time.perf_counter())
        return np.diff(t), sum(tree["n_nodes"] for tree in trees)

    def run(n):
        rows, nodes = [], 0
        for _ in range(n):
            dt, nodes = one_step()
            rows.append(dt)
        rows = np.array(rows)
        return rows, nodes

    rows, nodes = run(n_steps)
    total = float(rows.sum())
    out = {"value": nodes * n_steps / total, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
           "sample": f"{n_steps} whole step(s) of the same workload and seed with {threads} BLAS thread(s), "
                     f"{total:.1f} s of CPU work; {total / n_steps * 1e3:.0f} ms per step on average, "
                     f"{rows.sum(axis=1).min() * 1e3:.0f} ms the best",
           "host_cpus": os.cpu_count(),
           "per_stage_ms_best": {"threads": int(threads),
                                 **{name: float(rows[:, i].min() * 1e3) for i, name in enumerate(stages)},
                                 "step": float(rows.sum(axis=1).min() * 1e3)}}
    if n_steps_one_thread > 0 and threadpool_limits is not None:
        with threadpool_limits(limits=1):
            rows1, _ = run(n_steps_one_thread)
        out["per_stage_ms_best_one_thread"] = {"threads": 1,
                                               **{name: float(rows1[:, i].min() * 1e3) for i, name in enumerate(stages)},
                                               "step": float(rows1.sum(axis=1).min() * 1e3)}
        out["sample"] += f"; then {n_steps_one_thread} step(s) with the BLAS held to one thread, {rows1.sum():.1f} s"
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2
    import torch
    import workloads
    import paper_2412_00061_amd as lib
    from paper_2412_00061_amd.binding import CTCSPEC_BF16, CTCSPEC_F32
    from workloads.device import dev_f32, dev_i32, dev_i64, to_device

    cfg = workloads.get_config(args.config if not args.config.isdigit() else int(args.config))
    torch.cuda.set_device(0)
    x = workloads.make_inputs(cfg, args.seed, args.variant)
    ctx = lib.Context.for_config(cfg)
    ctx.defer_topk_merge(args.deferred_merge)
    B, T, k, N, H, dh = cfg.B, cfg.T, cfg.k, cfg.max_nodes, cfg.H, cfg.dh
    scale = 1.0 / math.sqrt(dh)
    dt = CTCSPEC_BF16 if cfg.dtype == "bf16" else CTCSPEC_F32

    d_hidden, d_bias, d_root = to_device(x.hidden, cfg.dtype), dev_f32(x.bias), dev_i32(x.root_token)
    w0 = to_device(x.w, cfg.dtype)
    d_w = [w0] + [w0.clone() for _ in range(args.w_copies - 1)]
    base = [to_device(a, cfg.dtype) for a in (x.q, x.k_tree, x.v_tree, x.k_cache, x.v_cache)]
    sets = [base] + [[t.clone() for t in base] for _ in range(args.kv_sets - 1)]
    d_off, d_len = dev_i64(x.kv_off), dev_i32(x.ctx_len)

    def i32(*shape):
        return torch.empty(shape, dtype=torch.int32, device="cuda")

    def f32(*shape):
        return torch.empty(shape, dtype=torch.float32, device="cuda")

    words = (N + 63) // 64
    topk_id, topk_logp, lse = i32(B, T, k), f32(B, T, k), f32(B, T)
    n_cand, cand_tokens, cand_len, cand_score, cand_leaf = i32(B), i32(B, cfg.beam, T), i32(B, cfg.beam), \
        f32(B, cfg.beam), i32(B, cfg.beam)
    n_nodes_d, node_token, node_parent, node_depth = i32(B), i32(B, N), i32(B, N), i32(B, N)
    anc_mask = torch.empty((B, N, words), dtype=torch.int64, device="cuda")
    out_attn = f32(B, H, N, dh)
    targets = torch.full((B, N), -1, dtype=torch.int32, device="cuda")
    accept_len, accept_nodes, accept_tokens, next_token = i32(B), i32(B, T + 1), i32(B, T + 1), i32(B)

    # the four C calls of one step, marshalled once per rotation slot (weights copy x buffer set)
    period = len(d_w) * len(sets) // math.gcd(len(d_w), len(sets))
    slots = []
    for i in range(period):
        w = d_w[i % len(d_w)]
        q, kt, vt, kc, vc = sets[i % len(sets)]
        slots.append((
            lib.prepared(ctx, "ctc_draft_topk", dt, d_hidden, w, d_bias, B, T, cfg.D, cfg.Vp1, k, topk_id,
                         topk_logp, lse, None),
            lib.prepared(ctx, "ctc_collapse_tree", topk_id, topk_logp, d_root, B, T, k, cfg.blank_id, cfg.beam,
                         N, n_cand, cand_tokens, cand_len, cand_score, cand_leaf, n_nodes_d, node_token,
                         node_parent, node_depth, anc_mask),
            lib.prepared(ctx, "tree_verify_attn", dt, q, kc, vc, d_off, d_len, cfg.kv_cap, kt, vt, n_nodes_d,
                         anc_mask, B, H, dh, N, scale, out_attn),
            lib.prepared(ctx, "accept_longest", n_nodes_d, node_token, node_parent, node_depth, targets, B, T,
                         N, accept_len, accept_nodes, accept_tokens, next_token),
        ))

    def step(i):
        c1, c2, c3, c4 = slots[i % period]
        c1(); c2(); c3(); c4()

    def step_with_events(i, ev):
        calls = slots[i % period]
        ev[0].record()
        for j in range(4):
            calls[j]()
            ev[j + 1].record()

    # one untimed step to learn the (deterministic) tree, then plant an accepted path so that the
    # acceptance walk does real work: the deepest node's root path is what the verifier "agrees" with
    step(0)
    torch.cuda.synchronize()
    n_nodes = n_nodes_d.cpu().numpy()
    parent, token, depth = node_parent.cpu().numpy(), node_token.cpu().numpy(), node_depth.cpu().numpy()
    tgt = np.full((B, N), -1, dtype=np.int32)
    for b in range(B):
        node = int(np.argmax(depth[b, :n_nodes[b]]))
        while node > 0:
            tgt[b, parent[b, node]] = token[b, node]
            node = parent[b, node]
    targets.copy_(torch.from_numpy(tgt))

    graph = None
    if args.graph:
        # capture `period` consecutive steps (each on its own weights copy / buffer set) into one HIP
        # graph; K must then be a multiple of the period
        if args.steps % period != 0:
            args.steps = max(period, args.steps // period * period)
        cap_stream = torch.cuda.Stream()
        ctx.set_stream(cap_stream)
        with torch.cuda.stream(cap_stream):
            for i in range(2):
                step(i)
            cap_stream.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=cap_stream):
                for i in range(period):
                    step(i)
        torch.cuda.synchronize()

    def run(n, first):
        if graph is not None:
            for _ in range(n // period):
                graph.replay()
        else:
            for i in range(n):
                step(first + i)

    if graph is not None:
        graph.replay()
    else:
        run(args.warmup, 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps, args.warmup)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    us_per_step = wall / args.steps * 1e6
    accepted = accept_len.cpu().numpy()

    # second pass with HIP events around every call (on the stream the kernels run on): per-call times
    if graph is not None:
        ctx.set_stream(torch.cuda.current_stream())
    n_ev = min(args.steps, 200)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(n_ev)]
    for i in range(n_ev):
        step_with_events(args.warmup + args.steps + i, evs[i])
    torch.cuda.synchronize()
    per_call = np.array([[e[j].elapsed_time(e[j + 1]) * 1e3 for j in range(4)] for e in evs])  # us
    call_us = per_call.mean(axis=0)
    call_med = np.median(per_call, axis=0)
    # third pass: the library records HIP events directly around the draft head's main kernel (on the
    # stream it is launched on); this is the launch duration the roofline figure uses
    ctx.profile_draft_head(True)
    head_kernel_us = []
    for i in range(n_ev):
        step(args.warmup + args.steps + n_ev + i)
        head_kernel_us.append(ctx.draft_head_kernel_ms() * 1e3)
    ctx.profile_draft_head(False)
    torch.cuda.synchronize()
    head_kernel_us = np.array(head_kernel_us)

    # the read-only streaming probe on the same weight copies, in the same run: what this GPU delivers to a kernel
    # that only reads the matrix (events around each launch, on the launch stream)
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    w_bytes = d_w[0].numel() * d_w[0].element_size()
    probe_calls = [lib.prepared(ctx, "ctcspec_stream_probe", w, w_bytes, sink) for w in d_w]
    for i in range(6):
        probe_calls[i % len(probe_calls)]()
    torch.cuda.synchronize()
    n_pr = 48
    pr_ev = [torch.cuda.Event(enable_timing=True) for _ in range(n_pr + 1)]
    pr_ev[0].record()
    for i in range(n_pr):
        probe_calls[i % len(probe_calls)]()
        pr_ev[i + 1].record()
    torch.cuda.synchronize()
    probe_us = float(np.median([pr_ev[i].elapsed_time(pr_ev[i + 1]) * 1e3 for i in range(n_pr)]))
    probe_bytes = w_bytes // (128 * 1024) * (128 * 1024)
    probe_gbps = probe_bytes / (probe_us * 1e-6) / 1e9

    # step time from the events of the second pass (first event to last event of each step)
    step_ev = np.array([e[0].elapsed_time(e[4]) * 1e3 for e in evs])

    # full-depth variant: the same step with the verification attention of EVERY layer of the base model,
    # each layer on its own K/V cache and Q/K_tree/V_tree (buffer set l for layer l), still one stream
    n_layers = args.attn_layers if args.attn_layers >= 0 else (cfg.n_layers if cfg.dtype == "bf16" else 0)
    full_depth = None
    if n_layers > 0:
        attn_calls = []
        for q, kt, vt, kc, vc in sets:
            attn_calls.append(lib.prepared(ctx, "tree_verify_attn", dt, q, kc, vc, d_off, d_len, cfg.kv_cap, kt, vt,
                                           n_nodes_d, anc_mask, B, H, dh, N, scale, out_attn))

        def full_step(i):
            c1, c2, _, c4 = slots[i % period]
            c1(); c2()
            for l in range(n_layers):
                attn_calls[(i * n_layers + l) % len(attn_calls)]()
            c4()

        for i in range(3):
            full_step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.full_depth_steps):
            full_step(3 + i)
        torch.cuda.synchronize()
        fd_us = (time.perf_counter() - t0) / args.full_depth_steps * 1e6

    # closed-step variant: the step plus the two calls that close it - the base model's LM head over the tree
    # nodes' hidden states (greedy token per node, another pass over a [V, D] matrix) between attention and
    # acceptance, and the history update afterwards
    closed = None
    if not args.no_closed_step and cfg.dtype == "bf16":
        g = torch.Generator(device="cuda").manual_seed(args.seed + 1)
        node_hidden = torch.randn((B, N, cfg.D), generator=g, device="cuda", dtype=torch.float32)
        node_hidden = (node_hidden / node_hidden.pow(2).mean(-1, keepdim=True).sqrt()).to(torch.bfloat16)
        wb0 = (torch.randn((cfg.V, cfg.D), generator=g, device="cuda", dtype=torch.float32) * 0.02).to(torch.bfloat16)
        w_base = [wb0] + [wb0.clone() for _ in range(max(1, args.w_copies // 2) - 1)]
        vh_targets, new_len = i32(B, N), i32(B)
        vh_calls = [lib.prepared(ctx, "verify_head_argmax", dt, node_hidden, wb, n_nodes_d, B, N, cfg.D, cfg.V,
                                 vh_targets, None) for wb in w_base]
        acc_call = lib.prepared(ctx, "accept_longest", n_nodes_d, node_token, node_parent, node_depth, vh_targets,
                                B, T, N, accept_len, accept_nodes, accept_tokens, next_token)
        commit_calls = [lib.prepared(ctx, "kv_commit", dt, kt, vt, accept_len, accept_nodes, T, d_off, d_len,
                                     cfg.kv_cap, B, H, dh, N, kc, vc, new_len) for (q, kt, vt, kc, vc) in sets]

        def closed_step(i):
            c1, c2, c3, _ = slots[i % period]
            c1(); c2(); c3()
            vh_calls[i % len(vh_calls)]()
            acc_call()
            commit_calls[i % len(sets)]()

        for i in range(5):
            closed_step(i)
        torch.cuda.synchronize()
        n_cs = max(24, min(args.steps, 96))
        t0 = time.perf_counter()
        for i in range(n_cs):
            closed_step(5 + i)
        torch.cuda.synchronize()
        cs_us = (time.perf_counter() - t0) / n_cs * 1e6
        cs_ev = [torch.cuda.Event(enable_timing=True) for _ in range(2 * n_cs)]
        for i in range(n_cs):
            c1, c2, c3, _ = slots[i % period]
            c1(); c2(); c3()
            cs_ev[2 * i].record()
            vh_calls[i % len(vh_calls)]()
            cs_ev[2 * i + 1].record()
            acc_call()
            commit_calls[i % len(sets)]()
        torch.cuda.synchronize()
        vh_us = float(np.median([cs_ev[2 * i].elapsed_time(cs_ev[2 * i + 1]) * 1e3 for i in range(n_cs)]))
        vh_bytes = cfg.V * cfg.D * 2 + B * N * cfg.D * 2 + B * N * 4  # one pass over the weights for any number of nodes
        closed = {"calls": "ctc_draft_topk, ctc_collapse_tree, tree_verify_attn, verify_head_argmax, accept_longest, "
                           "kv_commit", "steps": n_cs, "us_per_step": cs_us,
                  "verify_head_argmax_us_median": vh_us, "verify_head_algorithmic_bytes": vh_bytes,
                  "verify_head_hbm_gbps": vh_bytes / (vh_us * 1e-6) / 1e9,
                  "verified_tokens_per_sec": int(n_nodes.sum()) / (cs_us * 1e-6)}

        # sampling-based acceptance on the same step: the head also writes its logits, one uniform number per node
        # draws the target's token from them, and the walk follows the drawn tokens
        if not args.no_sampled_acceptance:
            vh_logits = torch.empty((B, N, cfg.V), dtype=torch.float32, device="cuda")
            drawn = i32(B, N)
            uni = torch.rand((B, N), generator=g, device="cuda", dtype=torch.float32)
            head_z = lib.prepared(ctx, "verify_head_argmax", dt, node_hidden, w_base[0], n_nodes_d, B, N, cfg.D, cfg.V,
                                  vh_targets, vh_logits)
            draw = lib.prepared(ctx, "verify_sample_tokens", vh_logits, n_nodes_d, uni, 1.0, B, N, cfg.V, drawn)
            walk = lib.prepared(ctx, "accept_longest", n_nodes_d, node_token, node_parent, node_depth, drawn,
                                B, T, N, accept_len, accept_nodes, accept_tokens, next_token)
            for _ in range(5):
                head_z(); draw(); walk()
            torch.cuda.synchronize()
            n_sa = 48
            sa_ev = [torch.cuda.Event(enable_timing=True) for _ in range(3 * n_sa)]
            for i in range(n_sa):
                sa_ev[3 * i].record()
                head_z()
                sa_ev[3 * i + 1].record()
                draw()
                sa_ev[3 * i + 2].record()
                walk()
            torch.cuda.synchronize()
            hz_us = float(np.median([sa_ev[3 * i].elapsed_time(sa_ev[3 * i + 1]) * 1e3 for i in range(n_sa)]))
            dr_us = float(np.median([sa_ev[3 * i + 1].elapsed_time(sa_ev[3 * i + 2]) * 1e3 for i in range(n_sa)]))
            dr_bytes = int(n_nodes.sum()) * cfg.V * 4
            closed["sampled_acceptance"] = {
                "calls": "verify_head_argmax (logits written), verify_sample_tokens, accept_longest",
                "verify_head_with_logits_us_median": hz_us, "verify_sample_tokens_us_median": dr_us,
                "verify_sample_algorithmic_bytes": dr_bytes, "verify_sample_gbps": dr_bytes / (dr_us * 1e-6) / 1e9,
                "extra_us_over_greedy": hz_us - vh_us + dr_us,
                "accepted_plus_bonus": (accept_len.cpu().numpy() + 1).tolist()}
            del vh_logits

    # draft-module variant: the transformer layer that produces the T slot states (its own weights and
    # cache, the base family's shape), then the step.  Weight copies rotate so that no pass finds its matrix in
    # a cache; the layer's workspace is allocated once.
    draft_layer = None
    if not args.no_draft_layer and cfg.dtype == "bf16" and cfg.D % 256 == 0 and B * T <= 16:
        D = cfg.D
        F = args.draft_layer_ffn if args.draft_layer_ffn > 0 else (D * 43 // 16 + 255) // 256 * 256
        g = torch.Generator(device="cuda").manual_seed(args.seed + 2)

        def rnd(*shape, scale=1.0):
            return (torch.randn(shape, generator=g, device="cuda", dtype=torch.float32) * scale).to(torch.bfloat16)

        n_wsets = 2
        wsets, keep = [], []
        for _ in range(n_wsets):
            tens = (1 + 0.1 * rnd(D).float()).to(torch.bfloat16), rnd(3 * D, D, scale=D ** -0.5), \
                rnd(D, D, scale=D ** -0.5), (1 + 0.1 * rnd(D).float()).to(torch.bfloat16), \
                rnd(2 * F, D, scale=D ** -0.5), rnd(D, F, scale=F ** -0.5)
            keep.append(tens)
            wsets.append(lib.layer_weights(*tens))
        x_in = rnd(B, T, D)
        ws = torch.empty(lib.draft_layer_workspace_bytes(B, T, D, H, F), dtype=torch.uint8, device="cuda")
        kn, vn = torch.empty((B, H, T, dh), dtype=torch.bfloat16, device="cuda"), torch.empty((B, H, T, dh), dtype=torch.bfloat16, device="cuda")
        slot_hidden = torch.empty((B, T, D), dtype=torch.bfloat16, device="cuda")
        dl_calls = []
        for i, wst in enumerate(wsets):
            q, kt, vt, kc, vc = sets[i % len(sets)]
            dl_calls.append(lib.prepared(ctx, "draft_layer_forward", dt, x_in, wst, d_len, kc, vc, d_off, d_len,
                                         cfg.kv_cap, B, T, D, H, F, 1e-6, 10000.0, ws, ws.numel(), None, kn, vn,
                                         slot_hidden, None))
        for i in range(4):
            dl_calls[i % n_wsets]()
        torch.cuda.synchronize()
        n_dl = max(24, min(args.steps, 96))
        dl_ev = [torch.cuda.Event(enable_timing=True) for _ in range(n_dl + 1)]
        dl_ev[0].record()
        for i in range(n_dl):
            dl_calls[i % n_wsets]()
            dl_ev[i + 1].record()
        torch.cuda.synchronize()
        dl_us = np.array([dl_ev[i].elapsed_time(dl_ev[i + 1]) * 1e3 for i in range(n_dl)])
        # with the step behind it
        t0 = time.perf_counter()
        for i in range(n_dl):
            c1, c2, c3, c4 = slots[i % period]
            dl_calls[i % n_wsets](); c1(); c2(); c3(); c4()
        torch.cuda.synchronize()
        dls_us = (time.perf_counter() - t0) / n_dl * 1e6
        w_bytes = 2 * (3 * D * D + D * D + 2 * F * D + D * F)
        kv_bytes = int(sum(2 * H * int(l) * dh * 2 for l in x.ctx_len))
        dl_bytes = w_bytes + kv_bytes + 2 * D * 2 + 6 * B * T * D * 2
        draft_layer = {"call": "draft_layer_forward", "shape": f"B={B} T={T} D={D} H={H} F={F} ctx={x.ctx_len.tolist()}",
                       "calls": n_dl, "us_per_call_median": float(np.median(dl_us)), "us_per_call_mean": float(dl_us.mean()),
                       "algorithmic_bytes": dl_bytes, "weight_bytes": w_bytes,
                       "hbm_gbps": dl_bytes / (float(np.median(dl_us)) * 1e-6) / 1e9,
                       "frac_of_hbm_peak": dl_bytes / (float(np.median(dl_us)) * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                       "layer_plus_step_us": dls_us,
                       "layer_plus_step_verified_tokens_per_sec": int(n_nodes.sum()) / (dls_us * 1e-6)}

    # Eq. 5 variant of the candidates' value: one more KB-sized call on the step's logits and candidates
    sum_score = None
    if not args.no_sum_score:
        with_logits = lib.ctc_draft_topk(ctx, d_hidden, d_w[0], d_bias, k, want_logits=True)
        ss_out = {"cand_logp_sum": torch.empty((B, cfg.beam), dtype=torch.float32, device="cuda"),
                  "cand_rank_sum": i32(B, cfg.beam)}
        ss_call = lib.prepared(ctx, "ctc_sum_score", with_logits["logits"], with_logits["lse"], cand_tokens, cand_len,
                               n_cand, B, T, cfg.Vp1, cfg.blank_id, cfg.beam, ss_out["cand_logp_sum"],
                               ss_out["cand_rank_sum"])
        for _ in range(5):
            ss_call()
        torch.cuda.synchronize()
        n_ss = 64
        ss_ev = [torch.cuda.Event(enable_timing=True) for _ in range(n_ss + 1)]
        ss_ev[0].record()
        for i in range(n_ss):
            ss_call()
            ss_ev[i + 1].record()
        torch.cuda.synchronize()
        ss_us = np.array([ss_ev[i].elapsed_time(ss_ev[i + 1]) * 1e3 for i in range(n_ss)])
        changed = int((ss_out["cand_rank_sum"].cpu().numpy() != np.arange(cfg.beam)[None, :]).sum()
                      - int((ss_out["cand_rank_sum"].cpu().numpy() < 0).sum()))
        sum_score = {"call": "ctc_sum_score", "us_per_call_median": float(np.median(ss_us)),
                     "candidates": n_cand.cpu().numpy().tolist(),
                     "candidates_whose_rank_differs_from_the_best_alignment_order": changed,
                     "bound": "latency (KB-sized: one wavefront per candidate, T dependent steps)"}

    # the training objective (Sec. 3.2) at two shapes: T frames per position against the next <= T tokens, for many
    # positions at once (bandwidth: each row of logits read once, its gradient row written once), and whole
    # sequences at the paper's maximum training length (the recursions' latency: two dependent passes over the frames)
    ctc_loss = None
    if not args.no_ctc_loss:
        ctc_loss = {}
        for tag, (nb, nt, nl) in {"per_position": (args.ctc_loss_positions, T, T), "whole_sequence": (4, 2048, 1024)}.items():
            gen = torch.Generator(device="cuda").manual_seed(args.seed + 17)
            z = torch.randn((nb, nt, cfg.Vp1), dtype=torch.float32, device="cuda", generator=gen) * 2.0
            lab = torch.randint(0, cfg.Vp1 - 1, (nb, nl), dtype=torch.int32, device="cuda", generator=gen)
            lab_len = torch.randint(1, nl + 1, (nb,), dtype=torch.int32, device="cuda", generator=gen)
            fr_len = torch.full((nb,), nt, dtype=torch.int32, device="cuda")
            ws = torch.empty(lib.ctc_loss_workspace_bytes(nb, nt, nl), dtype=torch.uint8, device="cuda")
            out_l = torch.empty((nb,), dtype=torch.float32, device="cuda")
            out_g = torch.empty_like(z)
            cl_call = lib.prepared(ctx, "ctc_loss", z, lab, lab_len, fr_len, nb, nt, cfg.Vp1, nl, cfg.blank_id, ws,
                                   ws.numel(), out_l, out_g)
            for _ in range(3):
                cl_call()
            torch.cuda.synchronize()
            n_cl = 10
            cl_ev = [torch.cuda.Event(enable_timing=True) for _ in range(n_cl + 1)]
            cl_ev[0].record()
            for i in range(n_cl):
                cl_call()
                cl_ev[i + 1].record()
            torch.cuda.synchronize()
            cl_us = float(np.median([cl_ev[i].elapsed_time(cl_ev[i + 1]) * 1e3 for i in range(n_cl)]))
            cl_bytes = nb * nt * cfg.Vp1 * 8
            rows_zero = float(out_g.sum(-1).abs().max())
            ctc_loss[tag] = {"call": "ctc_loss", "shape": f"B={nb} T={nt} V+1={cfg.Vp1} Lmax={nl}", "us_per_call_median": cl_us,
                             "frames_per_sec": nb * nt / (cl_us * 1e-6), "algorithmic_bytes": cl_bytes,
                             "hbm_gbps": cl_bytes / (cl_us * 1e-6) / 1e9,
                             "frac_of_hbm_peak": cl_bytes / (cl_us * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                             "finite_losses": int(torch.isfinite(out_l).sum()), "max_abs_gradient_row_sum": rows_zero}
            del z, out_g, ws
        torch.cuda.empty_cache()

    # A/B of the tree layout: the paper's literal one (raw candidates at full length, removed positions masked)
    # under the same node cap, against the collapsed tree the step uses.  Statistics only; same kernel otherwise.
    literal = None
    if not args.no_literal_layout:
        raw_out = lib.ctc_raw_tree(ctx, topk_id, topk_logp, d_root, cfg.blank_id, cfg.beam, N)
        raw_call = lib.prepared(ctx, "ctc_raw_tree", topk_id, topk_logp, d_root, B, T, k, cfg.blank_id, cfg.beam, N,
                                *(raw_out[n_] for n_ in ("n_cand", "cand_tokens", "cand_len", "cand_score", "cand_leaf",
                                                         "n_nodes", "node_token", "node_parent", "node_depth",
                                                         "anc_mask", "node_removed")))
        for _ in range(5):
            raw_call()
        torch.cuda.synchronize()
        rt_ev = [torch.cuda.Event(enable_timing=True) for _ in range(65)]
        rt_ev[0].record()
        for i in range(64):
            raw_call()
            rt_ev[i + 1].record()
        torch.cuda.synchronize()
        rt_us = float(np.median([rt_ev[i].elapsed_time(rt_ev[i + 1]) * 1e3 for i in range(64)]))
        r_tok, r_leaf, r_rem, r_nn = (raw_out[n_].cpu().numpy() for n_ in ("cand_tokens", "cand_leaf", "node_removed",
                                                                           "n_nodes"))
        c_leaf, c_nc = cand_leaf.cpu().numpy(), n_cand.cpu().numpy()
        drafts_raw, drafts_col = [], []
        for b in range(B):
            seen = set()
            for c in range(cfg.beam):
                if r_leaf[b, c] < 0:
                    continue
                y, prev = [], None
                for tok in r_tok[b, c]:
                    if tok != cfg.blank_id and tok != prev:
                        y.append(int(tok))
                    prev = tok
                if y:
                    seen.add(tuple(y))
            drafts_raw.append(len(seen))
            drafts_col.append(int((c_leaf[b, :c_nc[b]] >= 0).sum()))
        literal = {"call": "ctc_raw_tree", "us_per_call_median": rt_us, "node_cap": N,
                   "nodes": r_nn.tolist(), "nodes_on_removed_positions": [(int((r_rem[b] == 1).sum())) for b in range(B)],
                   "distinct_drafts_whole_in_the_tree": drafts_raw,
                   "collapsed_layout_distinct_drafts_whole_in_the_tree": drafts_col,
                   "collapsed_layout_nodes": n_nodes.tolist()}

    head_b, attn_b, total_b = algorithmic_bytes(cfg, x.ctx_len, n_nodes)
    if n_layers > 0:
        fd_bytes = total_b + (n_layers - 1) * attn_b
        full_depth = {"attention_layers": n_layers, "distinct_kv_sets": len(sets), "steps": args.full_depth_steps,
                      "us_per_step": fd_us, "algorithmic_bytes": fd_bytes,
                      "hbm_gbps": fd_bytes / (fd_us * 1e-6) / 1e9,
                      "frac_of_hbm_peak": fd_bytes / (fd_us * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                      "verified_tokens_per_sec": int(n_nodes.sum()) / (fd_us * 1e-6)}
    head_us = float(head_kernel_us.mean())
    achieved = head_b / (head_us * 1e-6) / 1e9
    nodes_total = int(n_nodes.sum())
    result = {
        "metric": "verified_tokens_per_sec",
        "value": nodes_total / (us_per_step * 1e-6),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": us_per_step / 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: one draft+verify step, B={B} D={cfg.D} V+1={cfg.Vp1} T={T} k={k} "
                               f"beam={cfg.beam} max_nodes={N} H={H} dh={dh} ctx={x.ctx_len.tolist()}",
                   "variant": args.variant, "seed": args.seed, "n_nodes": n_nodes.tolist(),
                   "accepted_plus_bonus": (accepted + 1).tolist(),
                   "w_copies": len(d_w), "kv_sets": len(sets), "launch": "hip_graph" if graph is not None else "eager",
                   "draft_head_merge": "deferred to the collapse/tree kernel's prologue" if args.deferred_merge else
                                       "in its own kernel"},
        "us_per_step": us_per_step,
        "step_algorithmic_bytes": total_b,
        "step_hbm_gbps": total_b / (us_per_step * 1e-6) / 1e9,
        "step_frac_of_hbm_peak": total_b / (us_per_step * 1e-6) / 1e9 / HBM_PEAK_GBPS,
        "per_call_us_mean": {"ctc_draft_topk": float(call_us[0]), "ctc_collapse_tree": float(call_us[1]),
                             "tree_verify_attn": float(call_us[2]), "accept_longest": float(call_us[3])},
        "per_call_us_median": {"ctc_draft_topk": float(call_med[0]), "ctc_collapse_tree": float(call_med[1]),
                               "tree_verify_attn": float(call_med[2]), "accept_longest": float(call_med[3])},
        "step_us_from_events": {"p10": float(np.percentile(step_ev, 10)), "median": float(np.median(step_ev)),
                                "p90": float(np.percentile(step_ev, 90)), "n": int(len(step_ev))},
        "attention_hbm_gbps": attn_b / (float(call_us[2]) * 1e-6) / 1e9,
        "full_depth_variant": full_depth,
        "closed_step_variant": closed,
        "draft_layer_variant": draft_layer,
        "sum_score_variant": sum_score,
        "literal_layout_variant": literal,
        "ctc_loss_variant": ctc_loss,
        "roofline": {"kernel": "lmhead_bf16_mfma_kernel (ctc_draft_topk)", "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": read_traffic_summary(), "algorithmic_bytes_per_launch": head_b,
                     "launch_us": head_us, "launch_us_median": float(np.median(head_kernel_us)),
                     # the same matrix through the read-only streaming probe, same run (launch to launch by events,
                     # so about 2 us of dispatch are inside): the achievable rate beside the nominal peak
                     "stream_probe_gbps": probe_gbps, "stream_probe_us": probe_us,
                     "frac_of_stream_probe": achieved / probe_gbps,
                     # the same kernel in the committed rocprofv3 trace (7B shape): begin-to-end by the profiler's
                     # clock, without the dispatch time that an event pair around one launch also spans
                     "kernel_trace_avg_us": read_kernel_trace_us() if cfg.name == "7b_ctx2048" else None,
                     "call_us_incl_merge_kernel": float(call_us[0])},
    }
    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, x, args.cpu_steps, args.cpu_steps_one_thread)
    print(json.dumps(result))
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
