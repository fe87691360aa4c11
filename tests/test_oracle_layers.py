"""Pins for the oracle's layer functions: brute-force loops, finite differences,
closed forms and torch's own conv/pool/autograd routines on the same inputs."""
import itertools
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import layers as L

DT = torch.float64


def _rand(*shape, seed=0):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(*shape, dtype=DT, generator=g)


def _conv_brute(x, w, b, stride, pad):
    n, c, h, wd = x.shape
    o, _, k, _ = w.shape
    ho = (h + 2 * pad - k) // stride + 1
    wo = (wd + 2 * pad - k) // stride + 1
    y = torch.zeros(n, o, ho, wo, dtype=DT)
    for ni, oi, i, j in itertools.product(range(n), range(o), range(ho), range(wo)):
        acc = float(b[oi])
        for ci, r, s in itertools.product(range(c), range(k), range(k)):
            hi, wi = i * stride + r - pad, j * stride + s - pad
            if 0 <= hi < h and 0 <= wi < wd:
                acc += float(x[ni, ci, hi, wi]) * float(w[oi, ci, r, s])
        y[ni, oi, i, j] = acc
    return y


CONV_CASES = [(3, 1, 1, 5, 6), (3, 2, 1, 6, 6), (1, 2, 0, 6, 4), (1, 1, 0, 3, 3), (3, 1, 0, 5, 5)]


@pytest.mark.parametrize("k,stride,pad,h,w", CONV_CASES)
def test_conv_forward_matches_seven_loops(k, stride, pad, h, w):
    x, wt, b = _rand(2, 3, h, w, seed=1), _rand(4, 3, k, k, seed=2), _rand(4, seed=3)
    y, _ = L.conv2d_fwd(x, wt, b, stride, pad)
    assert torch.allclose(y, _conv_brute(x, wt, b, stride, pad), rtol=0, atol=1e-12)
    assert torch.allclose(y, F.conv2d(x, wt, b, stride=stride, padding=pad), rtol=0, atol=1e-12)


def _fd(fn, x, eps=1e-6):
    g = torch.zeros_like(x)
    flat, gf = x.view(-1), g.view(-1)
    for i in range(flat.numel()):
        old = float(flat[i])
        flat[i] = old + eps
        up = float(fn())
        flat[i] = old - eps
        dn = float(fn())
        flat[i] = old
        gf[i] = (up - dn) / (2 * eps)
    return g


@pytest.mark.parametrize("k,stride,pad,h,w", CONV_CASES)
def test_conv_backward_finite_differences_and_autograd(k, stride, pad, h, w):
    x, wt, b = _rand(2, 3, h, w, seed=4), _rand(4, 3, k, k, seed=5), _rand(4, seed=6)
    y, saved = L.conv2d_fwd(x, wt, b, stride, pad)
    r = _rand(*y.shape, seed=7)  # loss = <r, y>
    dx, dw, db = L.conv2d_bwd(r, saved, wt, stride, pad)
    f = lambda: (L.conv2d_fwd(x, wt, b, stride, pad)[0] * r).sum()
    assert torch.allclose(dx, _fd(f, x), rtol=1e-6, atol=1e-7)
    assert torch.allclose(dw, _fd(f, wt), rtol=1e-6, atol=1e-7)
    assert torch.allclose(db, _fd(f, b), rtol=1e-6, atol=1e-7)
    xa, wa, ba = (t.clone().requires_grad_() for t in (x, wt, b))
    (F.conv2d(xa, wa, ba, stride=stride, padding=pad) * r).sum().backward()
    assert torch.allclose(dx, xa.grad, atol=1e-12)
    assert torch.allclose(dw, wa.grad, atol=1e-12)
    assert torch.allclose(db, ba.grad, atol=1e-12)


def test_conv_backward_without_dx_returns_same_weight_grads():
    x, wt, b = _rand(2, 3, 5, 5, seed=8), _rand(4, 3, 3, 3, seed=9), _rand(4, seed=10)
    y, saved = L.conv2d_fwd(x, wt, b, 1, 1)
    r = _rand(*y.shape, seed=11)
    _, dw, db = L.conv2d_bwd(r, saved, wt, 1, 1)
    dx2, dw2, db2 = L.conv2d_bwd(r, saved, wt, 1, 1, need_dx=False)
    assert dx2 is None and torch.equal(dw, dw2) and torch.equal(db, db2)


def test_linear_matches_matrix_definition_and_autograd():
    x, wt, b = _rand(5, 7, 1, 1, seed=1), _rand(3, 7, seed=2), _rand(3, seed=3)
    y, saved = L.linear_fwd(x, wt, b)
    brute = torch.tensor([[float(b[o]) + sum(float(x[n, c, 0, 0]) * float(wt[o, c]) for c in range(7))
                           for o in range(3)] for n in range(5)], dtype=DT)
    assert torch.allclose(y.view(5, 3), brute, atol=1e-13)
    r = _rand(5, 3, 1, 1, seed=4)
    dx, dw, db = L.linear_bwd(r, saved, wt)
    xa, wa, ba = (t.clone().requires_grad_() for t in (x, wt, b))
    (F.linear(xa.view(5, 7), wa, ba) * r.view(5, 3)).sum().backward()
    assert torch.allclose(dx, xa.grad, atol=1e-13)
    assert torch.allclose(dw, wa.grad, atol=1e-13)
    assert torch.allclose(db, ba.grad, atol=1e-13)


def test_relu_derivative_is_zero_at_zero():
    x = torch.tensor([-1.0, 0.0, 2.0], dtype=DT)
    y, m = L.relu_fwd(x)
    assert y.tolist() == [0.0, 0.0, 2.0]
    assert L.relu_bwd(torch.ones(3, dtype=DT), m).tolist() == [0.0, 0.0, 1.0]


def test_maxpool_matches_loops_and_library():
    x = _rand(2, 3, 6, 4, seed=5)
    y, saved = L.maxpool2_fwd(x)
    for n, c, i, j in itertools.product(range(2), range(3), range(3), range(2)):
        win = [float(x[n, c, 2 * i + a, 2 * j + b]) for a in range(2) for b in range(2)]
        assert float(y[n, c, i, j]) == max(win)
    assert torch.equal(y, F.max_pool2d(x, 2))
    r = _rand(*y.shape, seed=6)
    dx = L.maxpool2_bwd(r, saved)
    xa = x.clone().requires_grad_()
    (F.max_pool2d(xa, 2) * r).sum().backward()
    assert torch.allclose(dx, xa.grad, atol=0)


def test_maxpool_tie_goes_to_first_in_row_major_order():
    x = torch.zeros(1, 1, 2, 2, dtype=DT)
    x[0, 0, 0, 1] = 3.0
    x[0, 0, 1, 0] = 3.0
    _, saved = L.maxpool2_fwd(x)
    dx = L.maxpool2_bwd(torch.ones(1, 1, 1, 1, dtype=DT), saved)
    assert dx.view(-1).tolist() == [0.0, 1.0, 0.0, 0.0]
    x0 = torch.zeros(1, 1, 2, 2, dtype=DT)
    _, saved0 = L.maxpool2_fwd(x0)
    assert L.maxpool2_bwd(torch.ones(1, 1, 1, 1, dtype=DT), saved0).view(-1).tolist() == [1.0, 0, 0, 0]


def test_gap_is_the_spatial_mean_and_spreads_gradient_evenly():
    x = _rand(2, 3, 4, 4, seed=7)
    y, saved = L.gap_fwd(x)
    assert torch.allclose(y.view(2, 3), x.view(2, 3, 16).sum(-1) / 16, atol=1e-15)
    d = L.gap_bwd(torch.ones(2, 3, 1, 1, dtype=DT), saved)
    assert torch.allclose(d, torch.full((2, 3, 4, 4), 1 / 16, dtype=DT))


def test_softmax_ce_closed_forms():
    # equal logits: loss = log(C); gradient = (1/C - onehot)/n
    z = torch.zeros(4, 10, 1, 1, dtype=DT)
    y = np.array([0, 3, 9, 3], dtype=np.int32)
    loss, dz = L.softmax_ce_fwd(z, y)
    assert abs(float(loss) - math.log(10)) < 1e-14
    assert abs(float(dz[1, 3]) - (0.1 - 1) / 4) < 1e-15 and abs(float(dz[1, 4]) - 0.1 / 4) < 1e-15
    # one dominant correct logit: loss -> 0
    z2 = torch.full((1, 10, 1, 1), -50.0, dtype=DT)
    z2[0, 7] = 50.0
    l2, _ = L.softmax_ce_fwd(z2, np.array([7]))
    assert float(l2) < 1e-30 + 1e-12
    # rows of the gradient sum to zero; matches finite differences and the library
    z3 = _rand(5, 10, 1, 1, seed=8)
    y3 = np.array([1, 2, 3, 4, 5])
    l3, d3 = L.softmax_ce_fwd(z3, y3)
    assert torch.allclose(d3.view(5, 10).sum(1), torch.zeros(5, dtype=DT), atol=1e-15)
    assert torch.allclose(d3, _fd(lambda: L.softmax_ce_fwd(z3, y3)[0], z3), atol=1e-8)
    assert abs(float(l3) - float(F.cross_entropy(z3.view(5, 10), torch.tensor(y3)))) < 1e-13
    # shift invariance incl. large logits (no overflow)
    l4, _ = L.softmax_ce_fwd(z3 + 1000.0, y3)
    assert abs(float(l4) - float(l3)) < 1e-9


# ------------------------------------------------------------------ batch normalisation
def test_batchnorm_forward_statistics_and_library_routine():
    g = torch.Generator().manual_seed(5)
    x = 3.0 + 2.0 * torch.randn(5, 6, 4, 3, dtype=DT, generator=g)
    gamma = 1.0 + 0.3 * torch.randn(6, dtype=DT, generator=g)
    beta = 0.2 * torch.randn(6, dtype=DT, generator=g)
    eps = 1e-5
    y, (xhat, rstd) = L.batchnorm_fwd(x, gamma, beta, eps)
    ref = F.batch_norm(x, None, None, gamma, beta, training=True, eps=eps)
    assert torch.allclose(y, ref, rtol=1e-12, atol=1e-12)
    # written out channel by channel from the definition (biased variance)
    for c in range(6):
        vals = x[:, c].reshape(-1)
        mu = vals.sum() / vals.numel()
        var = ((vals - mu) ** 2).sum() / vals.numel()
        expect = gamma[c] * (x[:, c] - mu) / torch.sqrt(var + eps) + beta[c]
        assert torch.allclose(y[:, c], expect, rtol=1e-12, atol=1e-12)
        # the output of a channel has mean beta and variance gamma^2 * var / (var + eps)
        assert abs(float(y[:, c].mean() - beta[c])) < 1e-12
        assert abs(float(y[:, c].var(unbiased=False) - gamma[c] ** 2 * var / (var + eps))) < 1e-12
    # invariant under a per-channel shift and (up to eps) scale of the input
    y2, _ = L.batchnorm_fwd(x + 7.0, gamma, beta, eps)
    assert torch.allclose(y, y2, rtol=1e-10, atol=1e-10)


def test_batchnorm_backward_autograd_finite_differences_and_orthogonality():
    g = torch.Generator().manual_seed(6)
    x = torch.randn(4, 3, 2, 5, dtype=DT, generator=g)
    gamma = 1.0 + 0.3 * torch.randn(3, dtype=DT, generator=g)
    beta = 0.2 * torch.randn(3, dtype=DT, generator=g)
    dy = torch.randn(4, 3, 2, 5, dtype=DT, generator=g)
    eps = 1e-3
    y, saved = L.batchnorm_fwd(x, gamma, beta, eps)
    dx, dgamma, dbeta = L.batchnorm_bwd(dy, saved, gamma)
    xa, ga, ba = (t.clone().requires_grad_() for t in (x, gamma, beta))
    F.batch_norm(xa, None, None, ga, ba, training=True, eps=eps).backward(dy)
    assert torch.allclose(dx, xa.grad, rtol=1e-10, atol=1e-12)
    assert torch.allclose(dgamma, ga.grad, rtol=1e-10, atol=1e-12)
    assert torch.allclose(dbeta, ba.grad, rtol=1e-10, atol=1e-12)
    # the input gradient of a channel is orthogonal to the constant, and to xhat up to the eps
    # term: sum dx*xhat = gamma * rstd * dgamma * eps / (var + eps)
    xhat, rstd = saved
    assert torch.allclose(dx.sum(dim=(0, 2, 3)), torch.zeros(3, dtype=DT), atol=1e-12)
    r = rstd.view(-1)
    assert torch.allclose((dx * xhat).sum(dim=(0, 2, 3)), gamma * r * dgamma * eps * r * r, rtol=1e-9, atol=1e-12)
    # central differences of sum(y * dy) with respect to single inputs and parameters
    h = 1e-6
    def f(xx, gg, bb):
        return float((L.batchnorm_fwd(xx, gg, bb, eps)[0] * dy).sum())
    for idx in [(0, 0, 0, 0), (3, 2, 1, 4), (1, 1, 0, 2)]:
        xp, xm = x.clone(), x.clone()
        xp[idx] += h
        xm[idx] -= h
        assert abs((f(xp, gamma, beta) - f(xm, gamma, beta)) / (2 * h) - float(dx[idx])) < 1e-6
    for c in range(3):
        e = torch.zeros(3, dtype=DT)
        e[c] = h
        assert abs((f(x, gamma + e, beta) - f(x, gamma - e, beta)) / (2 * h) - float(dgamma[c])) < 1e-6
        assert abs((f(x, gamma, beta + e) - f(x, gamma, beta - e)) / (2 * h) - float(dbeta[c])) < 1e-6


def test_round_bf16_is_round_to_nearest_even_on_the_upper_sixteen_bits():
    """Pins of the storage rounding used by the oracle's diagnostic mode: hand-worked values (bf16 keeps
    8 significand bits, so the spacing in [1, 2) is 2^-7 and a tie sits at odd multiples of 2^-8) and the
    bit-pattern definition on random values of every magnitude."""
    r = lambda v: float(L.round_bf16(torch.tensor([v], dtype=DT))[0])
    assert r(1.0) == 1.0
    assert r(1 + 2.0 ** -8) == 1.0                      # tie -> even (significand ...0)
    assert r(1 + 3 * 2.0 ** -8) == 1 + 2.0 ** -6        # tie -> even (1 + 2/128 -> significand ...10)
    assert r(1 + 2.0 ** -8 + 2.0 ** -20) == 1 + 2.0 ** -7   # just above the tie -> up
    assert r(-1 - 2.0 ** -8) == -1.0
    assert r(0.0) == 0.0 and r(3.0) == 3.0 and r(-0.15625) == -0.15625
    assert r(1 + 2.0 ** -8 + 2.0 ** -40) == 1.0         # the fp32 step comes first: 2^-40 is lost, then the tie goes to even
    g = torch.Generator().manual_seed(9)
    x = torch.randn(200000, dtype=DT, generator=g) * torch.exp(8 * torch.randn(200000, dtype=DT, generator=g))
    bits = x.to(torch.float32).view(torch.int32).to(torch.int64) & 0xFFFFFFFF
    want = ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16) << 16
    want = torch.where(want >= 2 ** 31, want - 2 ** 32, want).to(torch.int32).view(torch.float32).to(DT)
    assert torch.equal(L.round_bf16(x), want)
    assert torch.equal(L.round_bf16(L.round_bf16(x)), L.round_bf16(x))   # idempotent
