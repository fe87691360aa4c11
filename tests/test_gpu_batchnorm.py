"""GPU parity of training-mode batch normalisation (statistics per data-group) inside the
decoupled step, against the CPU oracle, on the residual networks in their standard form."""
import numpy as np
import pytest

from dds_inputs import workload
from dds_inputs.configs import ring_mixing, tiny_cnn, tiny_resnet
from parity import bf16_round, check_parity, flat_init, rel_errors, run_hip, run_oracle, tensor_slices, thresholds

pytestmark = pytest.mark.gpu

# bf16 storage makes a deep normalised net chaotic at the level of single bf16 steps (tests/parity.py header;
# measured on the oracle in tests/test_parity_sensitivity.py): per-tensor bounds of 0.5 against the exact oracle
# and 0.4 against its storage-rounding mode are what any two correct bf16 implementations can be held to there.
# The tight checks of the normalisation kernels are the fp32 runs below (1e-3 of the update on toy nets, 2e-2 at
# the ResNet-18 shapes) and the shallow bf16 net, which matches the rounding mode to 1e-3.
# A convolution bias that feeds a normalisation has an exactly zero gradient in exact arithmetic
# (the normalisation removes any per-channel constant): the oracle leaves it at ~1e-17, fp32 /
# bf16 arithmetic at rounding-noise level, so a ratio of the two says nothing. Those tensors are
# held to an absolute bound instead.
DEAD_BIAS_ABS = {"f32": 2e-6, "bf16": 2e-3}


def _dead_biases(wl, k0):
    ops = wl.ops[wl.bounds[k0]:wl.bounds[k0 + 1]]
    return {f"{i}.conv.bias" for i, op in enumerate(ops)
            if op["op"] == "conv" and i + 1 < len(ops) and ops[i + 1]["op"] == "bn"}


def _compare(wl, seed, T, every_step=True, tiny=False, shallow=False):
    print(f"[bn] {wl.name} K={wl.K} W={wl.W} B={wl.B} {wl.precision} T={T} seed={seed}", flush=True)
    hip, hl = run_hip(wl, seed, T, None, every_step)
    init = flat_init(wl, seed)
    dead = set().union(*[_dead_biases(wl, k0) for k0 in range(wl.K)])
    for mode, kw in thresholds(wl.precision, tiny, bn=not shallow):
        orc, ol = run_oracle(wl, seed, T, None, every_step, q=bf16_round() if mode == "rounded" else None)
        check_parity(wl, hip, orc, init, label=" bn " + mode, skip=dead, **kw)
        for hp, op in zip(hip, orc):
            for k0 in range(wl.K):
                for name, sl in tensor_slices(wl, k0):
                    if name in _dead_biases(wl, k0):
                        err = float(np.abs(hp[k0][sl] - op[k0][sl]).max())
                        assert err <= DEAD_BIAS_ABS[wl.precision], f"module {k0} {name}: abs {err:.3e}"
        loss_tol = 10 * kw["tol"]
        for t, (a, b) in enumerate(zip(hl, ol)):
            assert (a is None) == (b is None)
            if a is not None:
                assert abs(a - b) <= max(loss_tol * abs(b), 1e-5), f"loss at t={t} ({mode} oracle): {a} vs {b}"


def test_tiny_resnet_bn_every_step_fp32():
    _compare(tiny_resnet(K=3, W=2, B=4, bn=True), seed=21, T=10, tiny=True)


def test_tiny_resnet_bn_single_module_single_group_fp32():
    _compare(tiny_resnet(K=1, W=1, B=6, bn=True), seed=22, T=5, tiny=True)


def test_channel_counts_off_the_eight_channel_grid_fp32():
    # 4 and 12 channels: fp32 rows whose last group of eight is half empty
    _compare(tiny_resnet(K=2, W=2, B=3, c=4, bn=True), seed=23, T=6, tiny=True)
    _compare(tiny_resnet(K=2, W=3, B=5, c=6, hw=6, bn=True), seed=24, T=6, tiny=True)


def test_normalisation_in_front_of_max_pooling_with_momentum_fp32():
    # conv - bn - relu - maxpool: the pooling backward masks by the normalised ReLU output; momentum 0.9
    _compare(tiny_cnn(K=2, W=2, B=4, bn=True), seed=30, T=8, tiny=True)


def test_shallow_cnn_bn_bf16_matches_the_storage_rounding_mode():
    # two convolutions, each followed by a normalisation: too few stored values for a bf16 step to differ, so the
    # library must land on the rounding mode within the bounds of nets without normalisation
    _compare(tiny_cnn(K=2, W=2, B=16, precision="bf16", bn=True), seed=31, T=8, shallow=True)


def test_tiny_resnet_bn_bf16():
    _compare(tiny_resnet(K=3, W=2, B=16, precision="bf16", bn=True), seed=25, T=10)


def test_resnet18_bn_reduced_batch_fp32_arithmetic():
    # full channel counts and image sizes (several row splits per normalisation) in fp32, where every
    # tensor is held to the update guard
    wl = workload("cfg2_resnet18_bn", B=3, precision="f32")
    _compare(wl, seed=29, T=2 * (wl.K - 1) + 4, every_step=False)


def test_resnet18_bn_reduced_batch_bf16():
    wl = workload("cfg2_resnet18_bn", B=4)
    _compare(wl, seed=26, T=2 * (wl.K - 1) + 8, every_step=False)


def test_paper_resnet20_bn_reduced_batch_bf16():
    wl = workload("paper_r20_S4K2_bn", B=9)
    _compare(wl, seed=27, T=2 * (wl.K - 1) + 8, every_step=False)


def test_bn_with_a_ring_mixing_matrix_fp32():
    """Per-data-group gamma / beta and statistics under a sparse communication graph."""
    import torch
    import paper_2509_05679_amd as P
    from dds_inputs import make_batch, make_params
    from oracle import fdg
    wl = tiny_resnet(K=2, W=3, B=4, bn=True)
    mixing, seed, T = ring_mixing(3, 0.25), 28, 8
    tr = P.Trainer(P.Spec.from_workload(wl, mixing), wl.W)
    init = make_params(wl, seed)
    for k0 in range(wl.K):
        tr.dds_set_params(k0, init[k0])
    pipe = fdg.Pipeline(wl.ops, wl.bounds, wl.W, init, wl.lr, wl.momentum, None, torch.tensor(mixing, dtype=torch.float64))
    pipe.keep_history = False
    for t in range(T):
        batches = [make_batch(wl, seed, t, s) for s in range(wl.W)]
        tr.dds_step([torch.from_numpy(x).cuda() for x, _ in batches], [torch.from_numpy(y).cuda() for _, y in batches])
        pipe.step(batches)
    torch.cuda.synchronize()
    finit = flat_init(wl, seed)
    for s in range(wl.W):
        hp = [tr.dds_get_params_replica(k0, s) for k0 in range(wl.K)]
        op = [np.concatenate([p.numpy().ravel() for p in pipe.w[s][k0]]) for k0 in range(wl.K)]
        for k0, name, rel in rel_errors(wl, hp, op, finit)[0]:
            assert rel <= 1e-4, f"data-group {s} module {k0} layer {name}: {rel:.3e}"
    assert abs(tr.dds_consensus_error() - fdg.consensus_error(pipe.w)) <= 1e-3 * fdg.consensus_error(pipe.w)
    tr.close()
