"""GPU test of ctc_draft_topk_noalloc, the entry point that allocates nothing: through the C ABI, against
ctc_draft_topk (same kernels, so every output must agree bit for bit: ids, log-probabilities, lse, logits), on calls
in a row that share the library's static scratch - a large head first, then smaller ones, whose partial results
overwrite only part of what the call before left behind.
"""
import ctypes

import numpy as np
import pytest
import torch

import workloads
from workloads.device import dev_f32, to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pkg():
    import paper_2412_00061_amd as m
    m.load_library()
    return m


def _outputs(B, T, k, Vp1, want_logits):
    out = {"topk_id": torch.full((B, T, k), -7, dtype=torch.int32, device="cuda"),
           "topk_logp": torch.full((B, T, k), float("nan"), device="cuda"),
           "lse": torch.full((B, T), float("nan"), device="cuda")}
    if want_logits:
        out["logits"] = torch.full((B, T, Vp1), float("nan"), device="cuda")
    return out


def _case(seed, B, T, D, Vp1, dtype):
    rng = np.random.Generator(np.random.PCG64(seed))
    hidden = workloads.round_to_storage(rng.standard_normal((B, T, D), dtype=np.float32), dtype)
    w = workloads.round_to_storage(rng.standard_normal((Vp1, D), dtype=np.float32) * 0.05, dtype)
    bias = rng.standard_normal(Vp1).astype(np.float32) * 0.1
    return to_device(hidden, dtype), to_device(w, dtype), dev_f32(bias)


def test_noalloc_against_the_oracle(pkg):
    """Two calls in a row, the second smaller, against the float64 oracle (logits 2e-3, ids exact on the kernel's own
    logits).  First in this file: run alone in a fresh process, this is the call that finds no context ever created."""
    import oracle
    from gpu_harness import rel_err_rms_floor
    stream = torch.cuda.current_stream()
    for (B, T, D, Vp1, k) in ((2, 8, 1024, 3001, 4), (1, 4, 512, 700, 2)):
        rng = np.random.Generator(np.random.PCG64(Vp1))
        hidden = workloads.round_to_storage(rng.standard_normal((B, T, D), dtype=np.float32), "bf16")
        w = workloads.round_to_storage(rng.standard_normal((Vp1, D), dtype=np.float32) * 0.05, "bf16")
        bias = rng.standard_normal(Vp1).astype(np.float32) * 0.1
        got = pkg.ctc_draft_topk_noalloc(stream, to_device(hidden, "bf16"), to_device(w, "bf16"), dev_f32(bias), k,
                                         out=_outputs(B, T, k, Vp1, True), want_logits=True)
        torch.cuda.synchronize()
        z = got["logits"].cpu().numpy()
        ref = oracle.draft_topk(hidden, w, bias, k)
        assert rel_err_rms_floor(z, ref["z"]) <= 2e-3
        assert np.array_equal(got["topk_id"].cpu().numpy(), oracle.topk_per_slot(z, k))
        logp_ref, lse_ref = oracle.log_softmax(z)
        tol = 2e-5 + 4 * float(np.spacing(np.float32(np.max(np.abs(z)))))
        assert np.max(np.abs(got["lse"].cpu().numpy() - lse_ref)) <= tol


# (B, T, D, V+1, k, dtype): streaming kernel with a large head, the same kernel on fewer rows and columns, the
# many-column tile kernel, the generic kernels - each after the other on the same scratch
SEQUENCE = [
    (1, 8, 4096, 32001, 4, "bf16"),
    (1, 5, 1024, 1500, 3, "bf16"),
    (8, 8, 1024, 4097, 4, "bf16"),
    (1, 2, 512, 129, 8, "bf16"),
    (2, 3, 48, 11, 5, "f32"),
    (1, 8, 4096, 32001, 4, "bf16"),
]


def test_noalloc_matches_context_call_on_consecutive_calls(pkg):
    stream = torch.cuda.current_stream()
    for i, (B, T, D, Vp1, k, dtype) in enumerate(SEQUENCE):
        print(f"ctc_draft_topk_noalloc case {i}: B={B} T={T} D={D} V+1={Vp1} k={k} {dtype}", flush=True)
        hidden, w, bias = _case(100 + i, B, T, D, Vp1, dtype)
        ctx = pkg.Context(max_batch=B, max_slots=T, max_topk=k, max_vocab_rows=Vp1, max_nodes=8, max_heads=1,
                          max_head_dim=16)
        want_logits = Vp1 <= 5000
        ref = pkg.ctc_draft_topk(ctx, hidden, w, bias, k, want_logits=want_logits)
        got = pkg.ctc_draft_topk_noalloc(stream, hidden, w, bias, k, out=_outputs(B, T, k, Vp1, want_logits),
                                         want_logits=want_logits)
        torch.cuda.synchronize()
        for name in ref:
            assert torch.equal(ref[name].view(torch.int32), got[name].view(torch.int32)), (i, name)
        assert int(got["topk_id"].min()) >= 0 and bool(torch.isfinite(got["topk_logp"]).all())
        # without a bias, right behind: the scratch still holds the call before
        ref2 = pkg.ctc_draft_topk(ctx, hidden, w, None, k)
        got2 = pkg.ctc_draft_topk_noalloc(stream, hidden, w, None, k, out=_outputs(B, T, k, Vp1, False))
        torch.cuda.synchronize()
        for name in ref2:
            assert torch.equal(ref2[name].view(torch.int32), got2[name].view(torch.int32)), (i, name, "no bias")
        ctx.close()


def test_noalloc_rejects_what_its_scratch_cannot_hold(pkg):
    lib = pkg.load_library()
    h = torch.zeros((1, 8, 64), device="cuda")
    w = torch.zeros((8, 64), device="cuda")  # the size check comes before any access: the row count is only claimed
    ids = torch.zeros((1, 8, 4), dtype=torch.int32, device="cuda")
    lp = torch.zeros((1, 8, 4), device="cuda")
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = lib.ctc_draft_topk_noalloc(None, 0, p(h), p(w), None, 1, 8, 64, 65537, 4, p(ids), p(lp), None, None)
    assert rc == -2 and b"65536" in lib.ctcspec_last_error(None)
    rc = lib.ctc_draft_topk_noalloc(None, 0, p(h), p(w), None, 9, 8, 64, 8, 4, p(ids), p(lp), None, None)
    assert rc == -2  # 72 columns
    rc = lib.ctc_draft_topk_noalloc(None, 0, None, p(w), None, 1, 8, 64, 8, 4, p(ids), p(lp), None, None)
    assert rc == -1
    torch.cuda.synchronize()
