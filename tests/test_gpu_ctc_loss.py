"""GPU parity of ctc_loss (Sec. 3.2: negative log of Eq. 5 and its gradient) against the oracle.

fp32 logits in.  The recursions run in fp32 log space with every frame's values held relative to the frame's
largest (offsets summed in double), and the occupancies of a frame are divided by their computed sum, so the error
does not grow with the number of frames: measured, the loss agrees to the last float digit or two and the gradient
to about 1e-5 of max(|entry|, rms) from 8 to 1300 frames.  The bars: loss 2e-6 relative (a few float ulps),
gradient 1e-4.  Rows of the gradient must sum to zero (1e-5), frames past frame_len and unreachable labels give
zeros, and a second call reproduces every bit.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from gpu_harness import rel_err_rms_floor
from workloads.device import dev_f32, dev_i32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pkg():
    import paper_2412_00061_amd as m
    m.load_library()
    return m


def _case(seed, B, T, C, Lmax, blank, repeat_heavy=False, scale=2.0):
    rng = np.random.Generator(np.random.PCG64(seed))
    logits = (rng.standard_normal((B, T, C), dtype=np.float32) * np.float32(scale))
    frame_len = rng.integers(max(1, T // 2), T + 1, size=B).astype(np.int32)
    frame_len[0] = T
    label_len = np.array([rng.integers(0, min(Lmax, int(f)) + 1) for f in frame_len], dtype=np.int32)
    label_len[0] = min(Lmax, T // 2)
    toks = [v for v in range(C) if v != blank]
    pool = toks[:3] if repeat_heavy else toks
    labels = rng.choice(pool, size=(B, Lmax)).astype(np.int32)
    return logits, labels, label_len, frame_len


def _check(pkg, seed, B, T, C, Lmax, blank, **kw):
    logits, labels, label_len, frame_len = _case(seed, B, T, C, Lmax, blank, **kw)
    ctx = pkg.Context(max_batch=max(B, 1), max_slots=8, max_topk=4, max_vocab_rows=max(C, 8), max_nodes=8, max_heads=1,
                      max_head_dim=8)
    print(f"ctc_loss seed={seed} B={B} T={T} V+1={C} Lmax={Lmax}", flush=True)
    args = (dev_f32(logits), dev_i32(labels), dev_i32(label_len), dev_i32(frame_len), blank)
    res = pkg.ctc_loss(ctx, *args)
    again = pkg.ctc_loss(ctx, *args)
    only_loss = pkg.ctc_loss(ctx, *args, want_grad=False)
    torch.cuda.synchronize()
    loss, grad = res["loss"].cpu().numpy(), res["grad"].cpu().numpy()
    assert torch.equal(res["loss"], again["loss"]) and torch.equal(res["grad"], again["grad"])
    assert torch.equal(res["loss"], only_loss["loss"])
    for b in range(B):
        Tb, L = int(frame_len[b]), int(label_len[b])
        ref_loss, ref_grad = oracle.ctc_loss_and_grad(logits[b, :Tb], tuple(int(v) for v in labels[b, :L]), blank)
        if math.isinf(ref_loss):
            assert math.isinf(loss[b]) and not grad[b].any()
            continue
        assert abs(loss[b] - ref_loss) <= 2e-6 * max(1.0, abs(ref_loss)), (b, loss[b], ref_loss)
        assert rel_err_rms_floor(grad[b, :Tb], ref_grad) <= 1e-4, (b, rel_err_rms_floor(grad[b, :Tb], ref_grad))
        assert np.max(np.abs(grad[b, :Tb].astype(np.float64).sum(-1))) <= 1e-5
        assert not grad[b, Tb:].any()
    ctx.close()


@pytest.mark.parametrize("seed,B,T,C,Lmax,blank,kw", [
    (0, 4, 8, 12, 8, 11, {}),                         # the draft slots' shape: 8 frames, at most 8 labels
    (1, 3, 40, 50, 16, 0, {}),                        # blank first in the vocabulary
    (2, 5, 24, 9, 12, 4, dict(repeat_heavy=True)),    # repeated tokens: blanks forced between, shared rows
    (3, 2, 96, 300, 40, 299, {}),                     # several states per thread's row in LDS
    (4, 2, 200, 64, 100, 63, dict(scale=1.0)),        # 201 states
    (5, 1, 6, 5, 6, 2, dict(repeat_heavy=True)),      # labels that cannot be reached
])
def test_ctc_loss_shapes(pkg, seed, B, T, C, Lmax, blank, kw):
    _check(pkg, seed, B, T, C, Lmax, blank, **kw)


def test_ctc_loss_vocabulary_size_of_the_head(pkg):
    """V+1 = 32001 symbols (odd: the rows start at every alignment), 8 frames per position as the draft head
    produces them."""
    _check(pkg, 7, 6, 8, 32001, 8, 32000)


@pytest.mark.parametrize("C", [2, 3, 4, 5, 7, 2049, 4100, 65536])
def test_ctc_loss_row_widths(pkg, C):
    """Widths around the 16-byte boundaries and the steps in loads per thread, up to the largest supported."""
    _check(pkg, 20 + C, 3, 5, C, 3, C - 1)


def test_ctc_loss_many_states(pkg):
    """1025 labels: 2051 states, three per thread; the float64 oracle takes a few seconds."""
    _check(pkg, 8, 1, 1300, 40, 1025, 39, scale=0.5)


def test_ctc_loss_rejects_bad_arguments(pkg):
    ctx = pkg.Context(max_batch=1, max_slots=8, max_topk=4, max_vocab_rows=8, max_nodes=8, max_heads=1, max_head_dim=8)
    z = dev_f32(np.zeros((1, 4, 6), dtype=np.float32))
    one = dev_i32(np.array([1], dtype=np.int32))
    with pytest.raises(pkg.CtcspecError, match="blank_id"):
        pkg.ctc_loss(ctx, z, dev_i32(np.zeros((1, 2), dtype=np.int32)), one, one, 6)
    with pytest.raises(pkg.CtcspecError, match="Lmax"):
        pkg.ctc_loss(ctx, z, dev_i32(np.zeros((1, 2048), dtype=np.int32)), one, one, 5)
    with pytest.raises(pkg.CtcspecError, match="workspace"):
        pkg.ctc_loss(ctx, z, dev_i32(np.zeros((1, 2), dtype=np.int32)), one, one, 5,
                     workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    wide = dev_f32(np.zeros((1, 1, 70000), dtype=np.float32))
    with pytest.raises(pkg.CtcspecError, match="registers"):
        pkg.ctc_loss(ctx, wide, dev_i32(np.zeros((1, 2), dtype=np.int32)), one, one, 5)
    ctx.close()


def test_ctc_loss_largest_label_capacity(pkg):
    """Lmax = 2047: four states per thread, the shorter ring of loads ahead."""
    _check(pkg, 9, 2, 600, 33, 2047, 32, scale=0.5)


@pytest.mark.parametrize("B,T,Lmax,picks", [(4096, 8, 8, 8), (4, 2048, 1024, 1)])
def test_ctc_loss_at_the_benchmark_shapes(pkg, B, T, Lmax, picks):
    """The two shapes bench.py times (V+1 = 32001), logits drawn on the device: sampled sequences against the oracle,
    and for all of them finite losses and gradient rows that sum to zero."""
    C, blank = 32001, 32000
    gen = torch.Generator(device="cuda").manual_seed(5)
    z = torch.randn((B, T, C), dtype=torch.float32, device="cuda", generator=gen) * 2.0
    labels = torch.randint(0, C - 1, (B, Lmax), dtype=torch.int32, device="cuda", generator=gen)
    label_len = torch.randint(1, Lmax + 1, (B,), dtype=torch.int32, device="cuda", generator=gen)
    frame_len = torch.full((B,), T, dtype=torch.int32, device="cuda")
    ctx = pkg.Context(max_batch=1, max_slots=8, max_topk=4, max_vocab_rows=C, max_nodes=8, max_heads=1, max_head_dim=8)
    print(f"ctc_loss bench shape B={B} T={T} Lmax={Lmax}", flush=True)
    res = pkg.ctc_loss(ctx, z, labels, label_len, frame_len, blank)
    torch.cuda.synchronize()
    # a label with a repeated token needs a blank in between and may not fit T frames: those are +inf with zero rows
    finite = torch.isfinite(res["loss"])
    assert int(finite.sum()) >= B * 3 // 4
    sums = res["grad"].sum(-1).abs().amax(-1)
    assert float(sums.max()) <= 2e-5
    assert not bool(res["grad"][~finite].any())
    step = max(1, B // picks)
    for b in range(0, B, step)[:picks]:
        L = int(label_len[b])
        ref_loss, ref_grad = oracle.ctc_loss_and_grad(z[b].cpu().numpy(), tuple(int(v) for v in labels[b, :L].cpu().numpy()), blank)
        got_loss, got_grad = float(res["loss"][b]), res["grad"][b].cpu().numpy()
        if math.isinf(ref_loss):
            assert math.isinf(got_loss) and not got_grad.any()
            continue
        assert abs(got_loss - ref_loss) <= 2e-6 * max(1.0, abs(ref_loss)), (b, got_loss, ref_loss)
        assert rel_err_rms_floor(got_grad, ref_grad) <= 1e-4, (b, rel_err_rms_floor(got_grad, ref_grad))
    del z, res
    torch.cuda.empty_cache()
    ctx.close()
