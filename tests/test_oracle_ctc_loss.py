"""CPU pins of the CTC loss oracle (Sec. 3.2): agreement with the forward-only Eq. 5 oracle (itself pinned by
brute force), forward = backward, torch's ctc_loss and autograd, finite differences, and gradient identities."""
import math

import numpy as np
import pytest
import torch

import oracle


def _logits(seed, T, C, scale=2.0):
    return np.random.default_rng(seed).standard_normal((T, C)) * scale


def _logp(z):
    return z - np.log(np.exp(z).sum(-1, keepdims=True))


@pytest.mark.parametrize("seed,T,C,y,blank", [(0, 5, 4, (1, 2), 0), (1, 8, 6, (3, 3, 1), 5), (2, 6, 3, (), 2),
                                              (3, 4, 5, (2, 0, 1, 3), 4), (4, 7, 4, (1,), 3)])
def test_forward_backward_and_the_forward_only_oracle(seed, T, C, y, blank):
    lp = _logp(_logits(seed, T, C))
    alpha, beta, total = oracle.ctc_alpha_beta(lp, y, blank)
    assert math.isclose(total, oracle.ctc_sequence_logprob(lp, y, blank), rel_tol=1e-12)
    # the same total from the backward side, and from any frame: sum_s alpha_t(s) beta_t(s) / p_t(z_s) = P
    z = [blank]
    for tok in y:
        z += [tok, blank]
    back = np.logaddexp(beta[0, 0], beta[0, 1]) if len(z) > 1 else beta[0, 0]
    assert math.isclose(back, total, rel_tol=1e-12)
    for t in range(T):
        terms = [alpha[t, s] + beta[t, s] - lp[t, z[s]] for s in range(len(z))]
        assert math.isclose(np.logaddexp.reduce(terms), total, rel_tol=1e-11)


@pytest.mark.parametrize("seed,T,C,L", [(0, 8, 11, 3), (1, 12, 7, 5), (2, 6, 5, 6), (3, 9, 6, 1), (4, 10, 4, 0)])
def test_against_torch_ctc_loss_and_autograd(seed, T, C, L):
    blank = C - 1
    rng = np.random.default_rng(seed + 100)
    y = tuple(int(v) for v in rng.integers(0, C - 1, size=L))
    z = _logits(seed, T, C)
    loss, grad = oracle.ctc_loss_and_grad(z, y, blank)
    tz = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    tl = torch.nn.functional.ctc_loss(torch.log_softmax(tz, -1)[:, None, :], torch.tensor([y], dtype=torch.long),
                                      torch.tensor([T]), torch.tensor([L]), blank=blank, reduction="sum")
    if math.isinf(float(tl.detach())):
        assert math.isinf(loss) and not grad.any()
        return
    tl.backward()
    assert math.isclose(loss, float(tl.detach()), rel_tol=1e-10)
    assert np.allclose(grad, tz.grad.numpy(), rtol=1e-8, atol=1e-10)


def test_gradient_by_finite_differences_and_identities():
    T, C, blank, y = 6, 5, 0, (2, 2, 4)
    z = _logits(9, T, C, scale=1.0)
    loss, grad = oracle.ctc_loss_and_grad(z, y, blank)
    eps = 1e-6
    for (t, v) in [(0, 0), (1, 2), (3, 4), (5, 1), (2, 3)]:
        zp, zm = z.copy(), z.copy()
        zp[t, v] += eps
        zm[t, v] -= eps
        num = (oracle.ctc_loss_and_grad(zp, y, blank)[0] - oracle.ctc_loss_and_grad(zm, y, blank)[0]) / (2 * eps)
        assert math.isclose(grad[t, v], num, rel_tol=1e-5, abs_tol=1e-8)
    # a shift of a frame's logits changes nothing: each frame's gradient sums to zero
    assert np.allclose(grad.sum(-1), 0.0, atol=1e-12)
    # tokens that are neither in the label nor the blank only receive the softmax term
    p = np.exp(_logp(z))
    assert np.allclose(grad[:, [1, 3]], p[:, [1, 3]], rtol=1e-12)
    # unreachable label: infinite loss, zero gradient
    loss2, grad2 = oracle.ctc_loss_and_grad(z[:3], (1, 1, 1), blank)
    assert math.isinf(loss2) and not grad2.any()
