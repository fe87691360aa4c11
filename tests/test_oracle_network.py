"""Pins for the oracle's per-module forward/backward: whole-network finite
differences and an autograd model assembled from torch's library routines."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from dds_inputs import make_batch, make_params
from dds_inputs.configs import tiny_cnn, tiny_mlp, tiny_resnet
from oracle import fdg, network as N

DT = torch.float64


def _autograd_net(ops, params, x, y):
    """Same network through torch's own conv2d/linear/max_pool2d + autograd."""
    ps = [p.clone().requires_grad_() for p in params]
    slots = N.param_slots(ops)
    h, stack = x, []
    for op, s in zip(ops, slots):
        k = op["op"]
        if k == "conv":
            h = F.conv2d(h, ps[s], ps[s + 1], stride=op["stride"], padding=op["pad"])
        elif k == "linear":
            h = F.linear(h.flatten(1), ps[s], ps[s + 1]).view(h.shape[0], -1, 1, 1)
        elif k == "bn":
            h = F.batch_norm(h, None, None, ps[s], ps[s + 1], training=True, eps=op["eps"])
        elif k == "relu":
            h = F.relu(h)
        elif k == "maxpool2":
            h = F.max_pool2d(h, 2)
        elif k == "gap":
            h = F.adaptive_avg_pool2d(h, 1)
        elif k == "res_begin":
            stack.append(h)
        elif k == "res_add":
            xin = stack.pop()
            sc = op["shortcut"]
            short = F.conv2d(xin, ps[s], ps[s + 1], stride=sc["stride"], padding=sc["pad"]) if sc else xin
            h = short + op["scale"] * h
        elif k == "softmax_ce":
            h = F.cross_entropy(h.flatten(1), torch.as_tensor(y, dtype=torch.int64))
    h.backward()
    return float(h.detach()), [p.grad for p in ps]


def _flat_params(wl, seed=0):
    mods = make_params(wl, seed)
    return [torch.as_tensor(p, dtype=DT) for m in mods for p in m]


def tiny_resnet_bn():
    return tiny_resnet(bn=True)


@pytest.mark.parametrize("make", [tiny_resnet, tiny_cnn, tiny_mlp, tiny_resnet_bn])
def test_whole_network_gradient_matches_autograd(make):
    wl = make()
    params = _flat_params(wl)
    # non-zero biases so that bias paths are exercised
    g = torch.Generator().manual_seed(3)
    params = [p if p.dim() > 1 else 0.1 * torch.randn(p.shape, dtype=DT, generator=g) for p in params]
    x, y = make_batch(wl, 0, 0, 0)
    x = torch.as_tensor(x, dtype=DT)
    dlog, saved, loss = N.forward(wl.ops, params, x, torch.as_tensor(y, dtype=torch.int64))
    _, grads = N.backward(wl.ops, params, saved, dlog, need_dx=False)
    ref_loss, ref = _autograd_net(wl.ops, params, x, y)
    assert abs(float(loss) - ref_loss) < 1e-12
    for g1, g2 in zip(grads, ref):
        assert torch.allclose(g1, g2, rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("bn", [False, True])
def test_whole_network_gradient_matches_finite_differences(bn):
    wl = tiny_resnet(K=1, B=2 + bn, hw=4, c=4, bn=bn)
    params = _flat_params(wl)
    x, y = make_batch(wl, 0, 0, 0)
    x = torch.as_tensor(x, dtype=DT)
    yl = torch.as_tensor(y, dtype=torch.int64)
    dlog, saved, _ = N.forward(wl.ops, params, x, yl)
    _, grads = N.backward(wl.ops, params, saved, dlog, need_dx=False)
    rng = np.random.default_rng(0)
    eps = 1e-6
    for j, p in enumerate(params):
        flat = p.view(-1)
        for i in rng.choice(flat.numel(), size=min(6, flat.numel()), replace=False):
            old = float(flat[i])
            flat[i] = old + eps
            up = float(N.forward(wl.ops, params, x, yl)[2])
            flat[i] = old - eps
            dn = float(N.forward(wl.ops, params, x, yl)[2])
            flat[i] = old
            fd = (up - dn) / (2 * eps)
            assert abs(fd - float(grads[j].view(-1)[i])) <= 1e-6 * max(1.0, abs(fd)), (j, i)


def test_module_split_composes_to_the_whole_network():
    """Running the K groups one after another (forward) and in reverse (backward,
    handing the input gradient up the line) equals the unsplit network."""
    wl = tiny_resnet(K=3)
    mods = [[torch.as_tensor(p, dtype=DT) for p in m] for m in make_params(wl, 1)]
    x, y = make_batch(wl, 1, 0, 0)
    grads, loss = fdg.definition_gradient(wl.ops, wl.bounds, mods, x, y)
    flat = [p for m in mods for p in m]
    ref_loss, ref = _autograd_net(wl.ops, flat, torch.as_tensor(x, dtype=DT), y)
    assert abs(float(loss) - ref_loss) < 1e-12
    for g1, g2 in zip([g for m in grads for g in m], ref):
        assert torch.allclose(g1, g2, rtol=1e-10, atol=1e-12)


def test_input_gradient_of_a_module_matches_autograd():
    wl = tiny_resnet(K=2)
    mods = [[torch.as_tensor(p, dtype=DT) for p in m] for m in make_params(wl, 2)]
    ops1 = wl.ops[wl.bounds[1]:]
    h = torch.randn(3, 8, 8, 8, dtype=DT, generator=torch.Generator().manual_seed(0))
    y = np.array([1, 5, 9])
    dlog, saved, _ = N.forward(ops1, mods[1], h, torch.as_tensor(y, dtype=torch.int64))
    dx, _ = N.backward(ops1, mods[1], saved, dlog, need_dx=True)
    ha = h.clone().requires_grad_()
    ps = [p.clone() for p in mods[1]]
    slots = N.param_slots(ops1)
    # reuse the autograd net with the input requiring grad
    hh, stack = ha, []
    for op, s in zip(ops1, slots):
        k = op["op"]
        if k == "conv":
            hh = F.conv2d(hh, ps[s], ps[s + 1], stride=op["stride"], padding=op["pad"])
        elif k == "linear":
            hh = F.linear(hh.flatten(1), ps[s], ps[s + 1]).view(hh.shape[0], -1, 1, 1)
        elif k == "relu":
            hh = F.relu(hh)
        elif k == "gap":
            hh = F.adaptive_avg_pool2d(hh, 1)
        elif k == "res_begin":
            stack.append(hh)
        elif k == "res_add":
            xin = stack.pop()
            sc = op["shortcut"]
            short = F.conv2d(xin, ps[s], ps[s + 1], stride=sc["stride"], padding=sc["pad"]) if sc else xin
            hh = short + op["scale"] * hh
        elif k == "softmax_ce":
            hh = F.cross_entropy(hh.flatten(1), torch.as_tensor(y, dtype=torch.int64))
    hh.backward()
    assert torch.allclose(dx, ha.grad, rtol=1e-10, atol=1e-13)


def test_bf16_quantised_normalisation_input_moves_upstream_gradients_by_percents():
    """Why the bf16 GPU parity tests of normalised nets do not hold single tensors to the update guard:
    the library stores the convolution output in bf16 before normalising it. Quantising just that one
    tensor in the oracle (everything else fp64) flips the ReLU decision of the elements whose normalised
    value is within the quantisation step of zero; each flip changes the back-propagated gradient by its
    full value there, so the weight gradients upstream move by percents while gamma / beta, which see
    the un-flipped incoming gradient, move by tenths of a percent."""
    from dds_inputs.configs import Workload, _bn, _conv, _linear, _relu
    from oracle import layers as L
    c = 64
    ops = [_conv(3, c), _relu(), _conv(c, c), _bn(c), _relu(), {"op": "gap"}, _linear(c, 10), {"op": "softmax_ce"}]
    wl = Workload(name="sens", ops=ops, bounds=[0, len(ops)], K=1, W=1, B=32, in_shape=(3, 8, 8), classes=10,
                  precision="bf16", lr=0.05, momentum=0.0, steps=1)
    params = [torch.as_tensor(p, dtype=DT) for p in make_params(wl, 1)[0]]
    x, y = make_batch(wl, 1, 0, 0)
    x, y = torch.as_tensor(x, dtype=DT), torch.as_tensor(y, dtype=torch.int64)

    def grads():
        dlog, saved, _ = N.forward(ops, params, x, y)
        return N.backward(ops, params, saved, dlog, need_dx=False)[1]

    exact = grads()
    plain = L.batchnorm_fwd
    try:
        L.batchnorm_fwd = lambda t, g, b, eps: plain(t.to(torch.float32).to(torch.bfloat16).to(DT), g, b, eps)
        quant = grads()
    finally:
        L.batchnorm_fwd = plain
    rel = [float((a - b).norm() / a.norm()) for a, b in zip(exact, quant)]
    conv0_w, conv2_w, gamma, beta = rel[0], rel[2], rel[4], rel[5]
    assert 5e-3 < conv2_w < 1e-1 and 5e-3 < conv0_w < 1e-1   # percents
    assert gamma < 5e-3 and beta < 1e-2                         # tenths of a percent
    assert conv2_w > 5 * gamma


def test_storage_rounding_mode_rounds_exactly_at_the_documented_points():
    """The diagnostic mode of oracle.network with a recording q: the sequence of rounded tensors (by
    shape) on a residual block with a projection shortcut, and q = identity leaves every result bit-equal
    to the exact mode."""
    from dds_inputs.configs import Workload, _conv, _linear, _relu
    c = 4
    ops = [_conv(3, c), _relu(),
           {"op": "res_begin"}, _conv(c, 2 * c, stride=2), _relu(), _conv(2 * c, 2 * c),
           {"op": "res_add", "scale": 0.5, "shortcut": {"cin": c, "cout": 2 * c, "k": 1, "stride": 2, "pad": 0}}, _relu(),
           {"op": "gap"}, _linear(2 * c, 10), {"op": "softmax_ce"}]
    wl = Workload(name="rp", ops=ops, bounds=[0, len(ops)], K=1, W=1, B=2, in_shape=(3, 8, 8), classes=10,
                  precision="bf16", lr=0.05, momentum=0.0, steps=1)
    params = [torch.as_tensor(p, dtype=DT) for p in make_params(wl, 1)[0]]
    x, y = make_batch(wl, 1, 0, 0)
    x, y = torch.as_tensor(x, dtype=DT), torch.as_tensor(y, dtype=torch.int64)
    seen = []

    def rec(t):
        seen.append(tuple(t.shape))
        return t

    dlog, saved, loss = N.forward(ops, params, x, y, q=rec)
    fwd = list(seen)
    assert fwd == [
        (2, 3, 8, 8),                       # module input
        (c, 3, 3, 3), (2, c, 8, 8),         # stem weight; stem output after bias + ReLU (one rounding)
        (2 * c, c, 3, 3), (2, 2 * c, 4, 4),       # conv1 weight; its output after ReLU
        (2 * c, 2 * c, 3, 3),                     # conv2 weight; its output is NOT stored on its own
        (2 * c, c, 1, 1), (2, 2 * c, 4, 4),       # projection weight and its stored output
        (2, 2 * c, 4, 4),                         # block output after scale + add + ReLU
        (2, 2 * c, 1, 1),                         # global average pool
        (10, 2 * c),                              # classifier weight; the logits stay exact
        (2, 10, 1, 1),                            # d loss / d logits
    ]
    seen.clear()
    dx, grads = N.backward(ops, params, saved, dlog, need_dx=True, q=rec)
    assert seen == [
        (10, 2 * c), (2, 2 * c, 1, 1),            # classifier weight; gradient w.r.t. the pooled features
        (2, 2 * c, 4, 4),                         # pool backward
        (2, 2 * c, 4, 4),                         # ... after the block output's ReLU mask (idempotent)
        (2 * c, c, 1, 1),                         # projection weight (its input gradient waits for the sum)
        (2 * c, 2 * c, 3, 3), (2, 2 * c, 4, 4),   # conv2 weight; gradient w.r.t. conv1's output
        (2, 2 * c, 4, 4),                         # ... after conv1's ReLU mask
        (2 * c, c, 3, 3),                         # conv1 weight; its input gradient is not rounded alone
        (2, c, 8, 8),                             # main + shortcut gradient summed at the block input: one rounding
        (2, c, 8, 8),                             # ... after the stem's ReLU mask
        (c, 3, 3, 3), (2, 3, 8, 8),               # stem weight; gradient w.r.t. the images
    ]
    # identity rounding = exact mode, bit for bit
    dlog0, saved0, loss0 = N.forward(ops, params, x, y)
    dx0, grads0 = N.backward(ops, params, saved0, dlog0, need_dx=True)
    assert float(loss) == float(loss0) and torch.equal(dx, dx0)
    assert all(torch.equal(a, b) for a, b in zip(grads, grads0))


def test_storage_rounding_mode_stays_within_the_bf16_update_guard_of_the_exact_mode():
    """bf16 storage moves the gradients of a small residual net by percents -- inside the bf16 update guard of
    the parity tests (0.15), far above fp32 rounding: the mode is neither a no-op nor a different method."""
    from oracle import layers as L
    wl = tiny_resnet(K=1, B=8, c=16)
    params = _flat_params(wl)
    x, y = make_batch(wl, 0, 0, 0)
    x, y = torch.as_tensor(x, dtype=DT), torch.as_tensor(y, dtype=torch.int64)
    d0, s0, l0 = N.forward(wl.ops, params, x, y)
    g0 = N.backward(wl.ops, params, s0, d0, need_dx=False)[1]
    d1, s1, l1 = N.forward(wl.ops, params, x, y, q=L.round_bf16)
    g1 = N.backward(wl.ops, params, s1, d1, need_dx=False, q=L.round_bf16)[1]
    rel = [float((a - b).norm() / a.norm()) for a, b in zip(g0, g1)]
    assert max(rel) < 0.15 and min(rel) > 1e-4, rel
    assert abs(float(l0) - float(l1)) < 1e-2 * float(l0)
