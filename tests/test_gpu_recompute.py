"""Activation policy "recompute" (dds_spec.activations): a module with delay d > 0 keeps only its input and
output per ring slot plus the parameters that forward pass used, and rebuilds the other saved tensors with a
second forward pass before the backward pass (Section 3.2: the backward pass at t uses activations and weights
of t - 2d). The method is unchanged, so (a) the result equals the oracle's like the default policy's, and
(b) it equals the default policy's bit for bit, the kernels being deterministic."""
from __future__ import annotations

import numpy as np
import pytest

from dds_inputs import make_batch, make_params, workload
from dds_inputs.configs import ring_mixing, tiny_cnn, tiny_resnet
from parity import check_parity, flat_init, run_hip, run_oracle, thresholds

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("wl,delays,T", [
    (tiny_resnet(K=2, W=2, B=4, bn=True), None, 10),
    (tiny_cnn(K=2, W=2, B=4), None, 10),
    # the last module is delayed too: its logits are rebuilt before the loss gradient is taken
    (tiny_resnet(K=2, W=2, B=2), [4, 2], 16),
])
def test_recompute_policy_matches_the_oracle(wl, delays, T):
    hip, hl = run_hip(wl, 41, T, delays=delays, every_step=True, activations="recompute")
    orc, ol = run_oracle(wl, 41, T, delays=delays, every_step=True)
    init = flat_init(wl, 41)
    dead = {f"{i}.conv.bias" for k0 in range(wl.K) for i, op in enumerate(wl.ops[wl.bounds[k0]:wl.bounds[k0 + 1]])
            if op["op"] == "conv" and wl.ops[wl.bounds[k0] + i + 1]["op"] == "bn"}  # identically zero gradient
    (_, th), = thresholds("f32", tiny=True)
    check_parity(wl, hip, orc, init, label=" recompute", skip=dead, **th)
    for a, b in zip(hl, ol):
        assert (a is None) == (b is None)
        if a is not None:
            assert abs(a - b) <= 1e-3 * abs(b) + 1e-6


@pytest.mark.parametrize("name,B,steps,mixing", [
    ("cfg2_resnet18", 16, 24, None),
    ("cfg2_resnet18_bn", 16, 24, None),
    ("cfg1_cnn", 16, 20, None),
    ("cfg3_resnet56", 4, 40, None),
    ("cfg2_resnet18", 8, 20, 0.25),  # one weight copy per data-group: the snapshots hold all of them
])
def test_recompute_policy_is_bit_identical_to_storing_every_activation(name, B, steps, mixing):
    import torch
    import paper_2509_05679_amd as P
    wl = workload(name, B=B)
    init = make_params(wl, 43)
    pool = 5
    xs = [[torch.from_numpy(make_batch(wl, 43, t, s)[0]).cuda() for s in range(wl.W)] for t in range(pool)]
    ys = [[torch.from_numpy(make_batch(wl, 43, t, s)[1]).cuda() for s in range(wl.W)] for t in range(pool)]
    Pm = None if mixing is None else ring_mixing(wl.W, mixing)

    def run(policy):
        spec = P.Spec.from_workload(wl, mixing=Pm, activations=policy)
        nbytes = P.dds_arena_bytes(spec, wl.K, wl.W)
        tr = P.Trainer(spec, wl.W)
        for k0 in range(wl.K):
            tr.dds_set_params(k0, init[k0])
        losses = []
        for t in range(steps):
            tr.dds_step(xs[t % pool], ys[t % pool])
            if t % 7 == 6 and t >= wl.K - 1:
                losses.append(tr.dds_get_loss())
        torch.cuda.synchronize()
        reps = range(wl.W) if Pm is not None else [0]
        out = [tr.dds_get_params_replica(k0, r) for k0 in range(wl.K) for r in reps]
        tr.close()
        return out, losses, nbytes

    stored, ls, nb_s = run("store")
    again, la, nb_r = run("recompute")
    if Pm is None:  # W weight copies at this small batch: the parameter snapshots outweigh the activations saved
        assert nb_r < nb_s
    assert ls == la
    for i, (a, b) in enumerate(zip(stored, again)):
        assert np.isfinite(a).all()
        assert np.array_equal(a, b), f"parameter block {i}"
