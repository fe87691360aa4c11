"""Full-size checks (the shapes bench.py times: 4 x 128 images, ResNet-18 widths) of the paths beyond
the exact-mean hot path, on what the oracle can compute one piece at a time: the loss of mini-batch 0
at the initial weights and the last module's first update (iteration K-1), which need one full-batch
forward and the last module's backward only."""
import numpy as np
import pytest

from dds_inputs import make_batch, make_params, workload
from dds_inputs.configs import ring_mixing
from parity import tensor_slices

pytestmark = pytest.mark.gpu


def _dead_biases(wl, k0):
    """Convolution biases in front of a normalisation: their gradient is exactly zero."""
    ops = wl.ops[wl.bounds[k0]:wl.bounds[k0 + 1]]
    return {f"{i}.conv.bias" for i, op in enumerate(ops)
            if op["op"] == "conv" and i + 1 < len(ops) and ops[i + 1]["op"] == "bn"}


def _first_update(wl, seed, mixing, update_tol, rel_tol):
    import torch
    from oracle import network as N
    import paper_2509_05679_amd as P
    K = wl.K
    tr = P.Trainer(P.Spec.from_workload(wl, mixing), wl.W)
    init = make_params(wl, seed)
    for k0 in range(K):
        tr.dds_set_params(k0, init[k0])
    for t in range(K):
        xs = [torch.from_numpy(make_batch(wl, seed, t, s)[0]).cuda() for s in range(wl.W)]
        ys = [torch.from_numpy(make_batch(wl, seed, t, s)[1]).cuda() for s in range(wl.W)]
        tr.dds_step(xs, ys)
    torch.cuda.synchronize()
    loss_hip = tr.dds_get_loss()
    last_hip = [tr.dds_get_params_replica(K - 1, s) for s in range(wl.W)]
    first_hip = tr.dds_get_params(0)
    delta_hip = tr.dds_consensus_error()
    tr.close()
    DT = torch.float64
    mods = [[torch.as_tensor(p, dtype=DT) for p in m] for m in init]
    losses, grads = [], []
    for s in range(wl.W):  # every data-group normalises over its own mini-batch
        x, y = make_batch(wl, seed, 0, s)
        h = torch.as_tensor(x, dtype=DT)
        for k0 in range(K - 1):
            h, _, _ = N.forward(wl.ops[wl.bounds[k0]:wl.bounds[k0 + 1]], mods[k0], h)
        ops = wl.ops[wl.bounds[K - 1]:]
        dlog, saved, loss = N.forward(ops, mods[K - 1], h, torch.as_tensor(y, dtype=torch.int64))
        _, g = N.backward(ops, mods[K - 1], saved, dlog, need_dx=True)
        losses.append(float(loss))
        grads.append(g)
    want_loss = float(np.mean(losses))
    assert abs(loss_hip - want_loss) <= 2e-2 * abs(want_loss), (loss_hip, want_loss)
    Pm = np.full((wl.W, wl.W), 1.0 / wl.W) if mixing is None else np.asarray(mixing, dtype=np.float64)
    init_last = np.concatenate([p.numpy().ravel() for p in mods[K - 1]])
    wants = []
    for s in range(wl.W):
        want = np.concatenate([(p - wl.lr * sum(Pm[s, r] * grads[r][j] for r in range(wl.W))).numpy().ravel()
                               for j, p in enumerate(mods[K - 1])])
        wants.append(want)
        for name, sl in tensor_slices(wl, K - 1):
            du = np.linalg.norm(want[sl] - init_last[sl])
            err = np.linalg.norm(last_hip[s][sl] - want[sl])
            if name in _dead_biases(wl, K - 1):
                assert err <= 2e-3, (s, name, err)
                continue
            nrm = np.linalg.norm(want[sl])
            if s == 0:
                print(f"[full] {wl.name} module {K-1} {name}: update-rel {err / max(du, 1e-30):.3e} rel {err / max(nrm, 1e-30):.3e}", flush=True)
            assert err <= update_tol * du or err <= rel_tol * nrm, (s, name, err, du, nrm)
    if mixing is not None:  # the disagreement after the first mixing step, layer by layer
        mean = sum(wants) / wl.W
        want_delta = max(np.linalg.norm(w[sl] - mean[sl]) for w in wants for _, sl in tensor_slices(wl, K - 1))
        assert abs(delta_hip - want_delta) <= 0.1 * want_delta, (delta_hip, want_delta)
    else:
        assert delta_hip == 0.0
    # module 0 has not received a gradient yet: bit-exact initial weights
    assert np.array_equal(first_hip, np.concatenate([p.ravel() for p in init[0]]))


def test_cfg2_full_size_ring_mixing_first_update():
    _first_update(workload("cfg2_resnet18"), seed=4, mixing=ring_mixing(4, 0.3), update_tol=1.5e-1, rel_tol=0.0)


def test_cfg2_bn_full_size_first_update_fp32_arithmetic():
    # the same shapes in fp32: every tensor within the update guard, i.e. what the bf16 run below loses is rounding
    _first_update(workload("cfg2_resnet18_bn", precision="f32"), seed=5, mixing=None, update_tol=2e-2, rel_tol=0.0)


def test_cfg2_bn_full_size_first_update():
    # bf16 with normalisation: ReLU decisions behind a bf16-quantised normalisation input differ from the fp64
    # oracle's for a fraction of a percent of the elements (see test_gpu_batchnorm.py), which moves upstream
    # gradients by up to ~16 % here; per tensor, the update guard or the stated bar relative to the parameter
    _first_update(workload("cfg2_resnet18_bn"), seed=5, mixing=None, update_tol=2.5e-1, rel_tol=2e-2)


def test_cfg2_full_size_long_run_properties():
    """Properties that hold at any size, at the shapes and in the launch configuration bench.py times (steps
    enqueued back to back on resident batches, so the module programs run ahead of each other): a module's
    weights are bit-exactly the initial ones until its first gradient arrives at iteration 2(K-1)-k0
    (Section 3.2: the gradient is defined as zero before that) and differ right after it; everything stays
    finite; and the stale-gradient iteration still descends: cycling over two fixed mini-batches per
    data-group at the configuration's step size, the loss (ln 10 at initialisation) falls steadily, by more than
    0.2 over 300 iterations."""
    import torch
    import paper_2509_05679_amd as P
    wl = workload("cfg2_resnet18")
    K, seed, pool = wl.K, 17, 2
    tr = P.Trainer(P.Spec.from_workload(wl), wl.W)
    init = make_params(wl, seed)
    flat = [np.concatenate([p.ravel() for p in m]) for m in init]
    for k0 in range(K):
        tr.dds_set_params(k0, init[k0])
    xs = [[torch.from_numpy(make_batch(wl, seed, t, s)[0]).cuda() for s in range(wl.W)] for t in range(pool)]
    ys = [[torch.from_numpy(make_batch(wl, seed, t, s)[1]).cuda() for s in range(wl.W)] for t in range(pool)]
    first = [2 * (K - 1) - k0 for k0 in range(K)]  # iteration of module k0's first update
    t = 0

    def advance(to):
        nonlocal t
        while t < to:
            tr.dds_step(xs[t % pool], ys[t % pool])
            t += 1

    for k0 in reversed(range(K)):  # first[] increases towards module 0
        advance(first[k0])        # iterations 0 .. first-1 done: no gradient yet
        assert np.array_equal(tr.dds_get_params(k0), flat[k0]), k0
        advance(first[k0] + 1)
        assert not np.array_equal(tr.dds_get_params(k0), flat[k0]), k0
    advance(K)
    loss0 = None
    losses = []
    while t < 300:
        advance(t + 25)
        losses.append(tr.dds_get_loss())
        loss0 = losses[0] if loss0 is None else loss0
    params = [tr.dds_get_params(k0) for k0 in range(K)]
    tr.close()
    print(f"[full] cfg2 long run: losses {['%.3f' % v for v in losses]}", flush=True)
    assert all(np.isfinite(p).all() for p in params)
    assert all(np.isfinite(losses))
    assert losses[-1] < losses[0] - 0.2, losses
    assert all(b < a + 0.01 for a, b in zip(losses, losses[1:])), losses
