"""Layer functions A_l and their chain-rule derivatives (Section 2.2, forward and
backward steps), written out from their definitions in fp64, NCHW.

Each forward returns (output, saved); each backward takes the gradient with
respect to the output and returns the gradient with respect to the input and
to the layer's weights. No fusion, no blocking: one tap of the convolution
stencil at a time.
"""
from __future__ import annotations

import torch

DT = torch.float64


def _taps(xp, k, stride, ho, wo):
    """Yield (r, s, view) where view[n,c,i,j] = xp[n,c,i*stride+r,j*stride+s]."""
    for r in range(k):
        for s in range(k):
            yield r, s, xp[:, :, r:r + stride * (ho - 1) + 1:stride, s:s + stride * (wo - 1) + 1:stride]


def conv_out_hw(h, w, k, stride, pad):
    return (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1


def conv2d_fwd(x, weight, bias, stride, pad):
    """y[n,o,i,j] = bias[o] + sum_{c,r,s} x[n,c,i*stride+r-pad,j*stride+s-pad] * weight[o,c,r,s]
    with x taken as zero outside its extent."""
    n, c, h, w = x.shape
    o, c2, k, k2 = weight.shape
    assert c == c2 and k == k2
    ho, wo = conv_out_hw(h, w, k, stride, pad)
    xp = torch.zeros((n, c, h + 2 * pad, w + 2 * pad), dtype=DT)
    xp[:, :, pad:pad + h, pad:pad + w] = x
    y = bias.view(1, o, 1, 1).expand(n, o, ho, wo).clone()
    for r, s, xs in _taps(xp, k, stride, ho, wo):
        y += torch.einsum("ncij,oc->noij", xs, weight[:, :, r, s])
    return y, (xp, x.shape)


def conv2d_bwd(dy, saved, weight, stride, pad, need_dx=True):
    """Derivatives of conv2d_fwd: (dx, dweight, dbias)."""
    xp, xshape = saved
    n, c, h, w = xshape
    o, _, k, _ = weight.shape
    ho, wo = dy.shape[2], dy.shape[3]
    dweight = torch.zeros_like(weight)
    dxp = torch.zeros_like(xp)
    for r, s, xs in _taps(xp, k, stride, ho, wo):
        dweight[:, :, r, s] = torch.einsum("noij,ncij->oc", dy, xs)
    if need_dx:
        for r, s, dxs in _taps(dxp, k, stride, ho, wo):
            dxs += torch.einsum("noij,oc->ncij", dy, weight[:, :, r, s])
    dbias = dy.sum(dim=(0, 2, 3))
    dx = dxp[:, :, pad:pad + h, pad:pad + w].clone() if need_dx else None
    return dx, dweight, dbias


def linear_fwd(x, weight, bias):
    """x is [N, cin, 1, 1]; y[n,o] = bias[o] + sum_c x[n,c] * weight[o,c]."""
    n = x.shape[0]
    x2 = x.reshape(n, -1)
    y = x2 @ weight.t() + bias
    return y.reshape(n, -1, 1, 1), (x2, x.shape)


def linear_bwd(dy, saved, weight, need_dx=True):
    x2, xshape = saved
    dy2 = dy.reshape(dy.shape[0], -1)
    dweight = dy2.t() @ x2
    dbias = dy2.sum(dim=0)
    dx = (dy2 @ weight).reshape(xshape) if need_dx else None
    return dx, dweight, dbias


def relu_fwd(x):
    y = torch.where(x > 0, x, torch.zeros_like(x))
    return y, (x > 0)


def relu_bwd(dy, mask):
    """d relu / dx = 1 for x > 0 and 0 otherwise (0 at x = 0)."""
    return torch.where(mask, dy, torch.zeros_like(dy))


def batchnorm_fwd(x, gamma, beta, eps):
    """Batch normalisation in training mode, the layer that follows every convolution in the
    standard definition of the ResNet-20 of the experiment section; a layer A_l(h, w_l) of
    Section 2.1 with w_l = (gamma, beta), evaluated on one data-group's mini-batch:
      mu[c]  = mean over (n, i, j) of x[n,c,i,j]
      var[c] = mean over (n, i, j) of (x[n,c,i,j] - mu[c])^2      (biased)
      xhat   = (x - mu) / sqrt(var + eps),   y = gamma[c] * xhat + beta[c]."""
    mu = x.mean(dim=(0, 2, 3), keepdim=True)
    var = ((x - mu) ** 2).mean(dim=(0, 2, 3), keepdim=True)
    rstd = 1.0 / torch.sqrt(var + eps)
    xhat = (x - mu) * rstd
    y = gamma.view(1, -1, 1, 1) * xhat + beta.view(1, -1, 1, 1)
    return y, (xhat, rstd)


def batchnorm_bwd(dy, saved, gamma):
    """Chain rule through batchnorm_fwd, mu and var included (m = N*H*W values per channel):
      dbeta = sum dy,  dgamma = sum dy * xhat,
      dx = gamma / sqrt(var + eps) * (dy - dbeta / m - xhat * dgamma / m)."""
    xhat, rstd = saved
    n, c, h, w = dy.shape
    m = n * h * w
    dbeta = dy.sum(dim=(0, 2, 3))
    dgamma = (dy * xhat).sum(dim=(0, 2, 3))
    dx = gamma.view(1, -1, 1, 1) * rstd * (dy - dbeta.view(1, -1, 1, 1) / m - xhat * dgamma.view(1, -1, 1, 1) / m)
    return dx, dgamma, dbeta


def maxpool2_fwd(x):
    """2x2 windows, stride 2. The selected element of a window is its first
    maximum in row-major order (strict comparisons)."""
    n, c, h, w = x.shape
    assert h % 2 == 0 and w % 2 == 0
    cand = [x[:, :, 0::2, 0::2], x[:, :, 0::2, 1::2], x[:, :, 1::2, 0::2], x[:, :, 1::2, 1::2]]
    best = cand[0].clone()
    arg = torch.zeros(best.shape, dtype=torch.int64)
    for q in range(1, 4):
        better = cand[q] > best
        best = torch.where(better, cand[q], best)
        arg = torch.where(better, torch.full_like(arg, q), arg)
    return best, (arg, x.shape)


def maxpool2_bwd(dy, saved):
    arg, xshape = saved
    dx = torch.zeros(xshape, dtype=DT)
    views = [dx[:, :, 0::2, 0::2], dx[:, :, 0::2, 1::2], dx[:, :, 1::2, 0::2], dx[:, :, 1::2, 1::2]]
    for q in range(4):
        views[q] += torch.where(arg == q, dy, torch.zeros_like(dy))
    return dx


def gap_fwd(x):
    return x.mean(dim=(2, 3), keepdim=True), x.shape


def gap_bwd(dy, xshape):
    n, c, h, w = xshape
    return (dy / (h * w)).expand(n, c, h, w).clone()


def softmax_ce_fwd(logits, labels):
    """Mean over the mini-batch of phi = -log softmax(logits)[label] (the mini-batch
    loss Phi of Section 2.1). Returns (loss, d loss / d logits)."""
    n = logits.shape[0]
    z = logits.reshape(n, -1)
    z = z - z.max(dim=1, keepdim=True).values
    logp = z - torch.log(torch.exp(z).sum(dim=1, keepdim=True))
    idx = torch.arange(n)
    lab = torch.as_tensor(labels, dtype=torch.int64)
    loss = -logp[idx, lab].mean()
    p = torch.exp(logp)
    p[idx, lab] -= 1.0
    return loss, (p / n).reshape(logits.shape)


def round_bf16(x):
    """Storage rounding of the diagnostic mode (oracle.network): the value as an fp32 number
    rounded to bfloat16 (8 significand bits: the upper 16 bits of the fp32 pattern) to
    nearest, ties to even, returned in fp64. The two conversions are the array library's;
    tests/test_oracle_layers.py pins them to the bit-pattern definition."""
    return x.to(torch.float32).to(torch.bfloat16).to(DT)
