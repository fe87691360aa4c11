"""Forward and backward pass of a contiguous group of layers g(k) = {p_k..q_k}
(Section 3.2), op by op, fp64.

`ops` is a list of op records (dicts with key "op": conv, linear, bn, relu, maxpool2,
gap, res_begin, res_add, softmax_ce); `params` is the flat list of that group's
weight tensors in canonical order (for each conv/linear/bn/projection-shortcut in op
order: weight, then bias; for bn: gamma, then beta).

Diagnostic storage-rounding mode. `forward` and `backward` take an optional `q`, a function
that rounds a tensor to a storage precision (tests pass round-to-nearest-even bf16). With
q = None (the default, and the contract the HIP library is held to) nothing below changes.
With q given, a value is rounded exactly where a mixed-precision implementation that keeps
activations, the forward/backward weight operand and inter-layer error gradients in that
storage precision would round it, and nowhere else:
  forward : the module input; the weight operand of every conv / linear / projection
            shortcut (biases and normalisation parameters stay exact); the output of every
            group  conv|linear [-> res_add] [-> relu]  and  bn [-> res_add] [-> relu]  (one
            rounding at the end of the group: bias, residual scale + add and ReLU happen on
            the exact accumulator); a conv output that feeds a bn; a projection shortcut's
            output; gap / maxpool outputs; d loss / d logits. Logits and the loss are exact.
  backward: the gradient w.r.t. every op input, after the ReLU mask of that input where
            there is one (masking and rounding commute) and after the sum at res_begin
            (the shortcut branch's gradient is added before the single rounding); the
            scaled gradient inside a residual branch (res_add) is not materialised.
Weight gradients, the update and the master weights are never rounded.
"""
from __future__ import annotations

from typing import List

import torch

from . import layers as L

DT = torch.float64


def param_slots(ops) -> List[int]:
    """Index of each op's weight tensor in the flat param list (-1 if it has none)."""
    slots, nxt = [], 0
    for op in ops:
        kind = op["op"]
        has = kind in ("conv", "linear", "bn") or (kind == "res_add" and op.get("shortcut"))
        slots.append(nxt if has else -1)
        if has:
            nxt += 2
    return slots


def n_params(ops) -> int:
    return sum(2 for s in param_slots(ops) if s >= 0)


def _rounds_after(ops, i):
    """Storage-rounding mode: is the output of op i stored (True) or consumed by an op fused
    behind it / kept exact (False)?"""
    kind = ops[i]["op"]
    nxt = ops[i + 1]["op"] if i + 1 < len(ops) else None
    if kind in ("conv", "linear"):
        return nxt not in ("res_add", "relu", "softmax_ce")   # logits stay exact
    if kind == "bn":
        return nxt not in ("res_add", "relu")
    if kind == "res_add":
        return nxt != "relu"
    return kind in ("relu", "gap", "maxpool2")


def forward(ops, params, x, labels=None, q=None):
    """Run the ops on x. Returns (output, saved, loss). If the last op is
    softmax_ce, output is d loss / d logits and loss is the mini-batch mean.
    q: optional storage rounding (see the module header)."""
    slots = param_slots(ops)
    saved = []
    res_stack = []
    h = x if q is None else q(x)
    loss = None
    wq = (lambda w: w) if q is None else q
    for i, (op, ps) in enumerate(zip(ops, slots)):
        kind = op["op"]
        if kind == "conv":
            h, sv = L.conv2d_fwd(h, wq(params[ps]), params[ps + 1], op["stride"], op["pad"])
        elif kind == "linear":
            h, sv = L.linear_fwd(h, wq(params[ps]), params[ps + 1])
        elif kind == "bn":
            h, sv = L.batchnorm_fwd(h, params[ps], params[ps + 1], op["eps"])
        elif kind == "relu":
            h, sv = L.relu_fwd(h)
        elif kind == "maxpool2":
            h, sv = L.maxpool2_fwd(h)
        elif kind == "gap":
            h, sv = L.gap_fwd(h)
        elif kind == "res_begin":
            res_stack.append(h)
            sv = None
        elif kind == "res_add":
            xin = res_stack.pop()
            sc = op.get("shortcut")
            if sc:
                short, sv = L.conv2d_fwd(xin, wq(params[ps]), params[ps + 1], sc["stride"], sc["pad"])
                short = wq(short)
            else:
                short, sv = xin, None
            h = short + op["scale"] * h
        elif kind == "softmax_ce":
            assert labels is not None
            loss, h = L.softmax_ce_fwd(h, labels)
            h = wq(h)
            sv = None
        else:
            raise ValueError(kind)
        if q is not None and _rounds_after(ops, i):
            h = q(h)
        saved.append(sv)
    assert not res_stack
    return h, saved, loss


def backward(ops, params, saved, dout, need_dx=True, q=None):
    """Chain rule through the ops in reverse. `dout` is the gradient with respect
    to the group's output (for a group ending in softmax_ce: the d loss / d logits
    that forward returned). Returns (dx, grads) with grads aligned to params.
    q: optional storage rounding (see the module header)."""
    slots = param_slots(ops)
    wq = (lambda w: w) if q is None else q
    grads = [None] * len(params)
    d = dout
    res_grad = []  # gradients waiting to be added at the matching res_begin
    first_weighted = next((i for i, s in enumerate(slots) if s >= 0), None)
    for i in range(len(ops) - 1, -1, -1):
        op, ps, sv = ops[i], slots[i], saved[i]
        kind = op["op"]
        # the gradient w.r.t. the group's input is needed unless this is the first
        # weighted op of a group whose caller asked for no dx
        want_dx = need_dx or i != first_weighted or bool(res_grad)
        if kind == "conv":
            d, grads[ps], grads[ps + 1] = L.conv2d_bwd(d, sv, wq(params[ps]), op["stride"], op["pad"], want_dx)
        elif kind == "linear":
            d, grads[ps], grads[ps + 1] = L.linear_bwd(d, sv, wq(params[ps]), want_dx)
        elif kind == "bn":
            d, grads[ps], grads[ps + 1] = L.batchnorm_bwd(d, sv, params[ps])
        elif kind == "relu":
            d = L.relu_bwd(d, sv)
        elif kind == "maxpool2":
            d = L.maxpool2_bwd(d, sv)
        elif kind == "gap":
            d = L.gap_bwd(d, sv)
        elif kind == "res_add":
            sc = op.get("shortcut")
            if sc:
                dshort, grads[ps], grads[ps + 1] = L.conv2d_bwd(d, sv, wq(params[ps]), sc["stride"], sc["pad"], True)
            else:
                dshort = d
            res_grad.append(dshort)
            d = op["scale"] * d
        elif kind == "res_begin":
            d = res_grad.pop() if d is None else d + res_grad.pop()
        elif kind == "softmax_ce":
            pass  # dout already is d loss / d logits
        else:
            raise ValueError(kind)
        if q is not None and d is not None and kind not in ("res_add", "softmax_ce"):
            # the gradient w.r.t. this op's input is stored, unless the op sits right behind a
            # res_begin: then the shortcut branch's gradient is added first (one rounding of the sum)
            if not (i > 0 and ops[i - 1]["op"] == "res_begin"):
                d = q(d)
    return d, grads
