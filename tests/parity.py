"""Shared helpers of the GPU parity tests: run the HIP library and the CPU oracle on
the same seeded workload and compare parameter trajectories tensor by tensor."""
from __future__ import annotations

import numpy as np

from dds_inputs import make_batch, make_params, param_shapes


def run_hip(wl, seed, T, delays=None, every_step=False, lr_schedule=None, activations="store"):
    import torch
    import paper_2509_05679_amd as P
    spec = P.Spec.from_workload(wl, activations=activations)
    tr = P.Trainer(spec, wl.W, delays)
    init = make_params(wl, seed)
    for k0 in range(wl.K):
        tr.dds_set_params(k0, init[k0])
    traj, losses = [], []
    for t in range(T):
        xs, ys = [], []
        for s in range(wl.W):
            x, y = make_batch(wl, seed, t, s)
            xs.append(torch.from_numpy(x).cuda())
            ys.append(torch.from_numpy(y).cuda())
        if lr_schedule is None:
            tr.dds_step(xs, ys)
        else:
            tr.dds_step(xs, ys, lr_schedule(t))
        torch.cuda.synchronize()
        try:
            losses.append(tr.dds_get_loss())
        except P.DdsError:
            losses.append(None)
        if every_step or t == T - 1:
            traj.append([tr.dds_get_params(k0) for k0 in range(wl.K)])
    tr.close()
    return traj, losses


def run_oracle(wl, seed, T, delays=None, every_step=False, lr_schedule=None):
    import torch
    from oracle import fdg
    pipe = fdg.Pipeline(wl.ops, wl.bounds, wl.W, make_params(wl, seed), wl.lr, wl.momentum, delays)
    pipe.keep_history = False
    traj, losses = [], []
    for t in range(T):
        if lr_schedule is not None:
            pipe.lr = lr_schedule(t)
        loss = pipe.step([make_batch(wl, seed, t, s) for s in range(wl.W)])
        losses.append(None if loss is None else float(loss))
        if every_step or t == T - 1:
            traj.append([np.concatenate([p.numpy().ravel() for p in pipe.w[0][k0]]) for k0 in range(wl.K)])
    return traj, losses


def tensor_slices(wl, k0):
    ops = wl.ops[wl.bounds[k0]:wl.bounds[k0 + 1]]
    out, off = [], 0
    for name, shape, _ in param_shapes(ops):
        n = int(np.prod(shape))
        out.append((name, slice(off, off + n)))
        off += n
    return out


def rel_errors(wl, hip_params, orc_params, init=None):
    """Relative L2 errors ||hip - oracle|| / ||oracle||.

    Returns (layer_rows, tensor_rows). A layer row groups a layer's weight and bias into
    the paper's layer weight vector w_l (Section 2.1: "the vectorization of the weight in
    the layer l"): (module, layer name, rel). A tensor row is per parameter tensor:
    (module, tensor name, rel on the parameter, rel on the update p(T) - p(0));
    the parameter ratio of a tensor the oracle leaves at exactly zero is 0 if the HIP side
    is exactly zero too and inf otherwise."""
    layer_rows, tensor_rows = [], []
    for k0 in range(wl.K):
        groups = {}
        for name, sl in tensor_slices(wl, k0):
            a, b = hip_params[k0][sl].astype(np.float64), orc_params[k0][sl]
            nb = np.linalg.norm(b)
            err = np.linalg.norm(a - b)
            rel = err / nb if nb > 0 else (0.0 if err == 0 else np.inf)
            upd = None
            if init is not None:
                i0 = init[k0][sl]
                du = np.linalg.norm(b - i0)
                # "no update yet": the oracle's fp64 mixing sum_r (1/S) w can move a weight by an ulp
                # of fp64 when 1/S is not a power of two, which is not an update to compare against
                floor = 1e-13 * max(np.linalg.norm(i0), 1.0)
                upd = (err / du) if du > floor else (0.0 if err <= floor else np.inf)
            tensor_rows.append((k0, name, rel, upd))
            g = groups.setdefault(name.rsplit(".", 1)[0], [0.0, 0.0])
            g[0] += err ** 2
            g[1] += nb ** 2
        for lname, (e2, n2) in groups.items():
            layer_rows.append((k0, lname, (e2 ** 0.5) / (n2 ** 0.5) if n2 > 0 else (0.0 if e2 == 0 else np.inf)))
    return layer_rows, tensor_rows


def flat_init(wl, seed):
    return [np.concatenate([p.ravel().astype(np.float64) for p in m]) for m in make_params(wl, seed)]
