"""GPU parity: the HIP library against the CPU oracle on the same seeded inputs.

Tolerances (tests/parity.py states them and what each is for): relative L2 per layer weight vector
against the exact fp64 oracle 1e-4 (fp32 path) / 2e-2 (bf16 path); per parameter tensor the error
relative to the accumulated update and an element-wise figure; on the bf16 path the latter two also,
tightly, against the oracle's storage-rounding mode.
"""
import math

import numpy as np
import pytest

from dds_inputs import workload
from dds_inputs.configs import odd_resnet, tiny_cnn, tiny_mlp, tiny_resnet, uneven_cnn
from parity import bf16_round, check_parity, flat_init, run_hip, run_oracle, thresholds

pytestmark = pytest.mark.gpu


def _compare(wl, seed, T, delays=None, every_step=False, lr_schedule=None, tiny=False):
    print(f"[parity] {wl.name} K={wl.K} W={wl.W} B={wl.B} {wl.precision} lr={wl.lr} mu={wl.momentum} T={T} seed={seed}",
          flush=True)
    hip, hl = run_hip(wl, seed, T, delays, every_step, lr_schedule)
    init = flat_init(wl, seed)
    worst = None
    for mode, kw in thresholds(wl.precision, tiny):
        orc, ol = run_oracle(wl, seed, T, delays, every_step, lr_schedule, q=bf16_round() if mode == "rounded" else None)
        w = check_parity(wl, hip, orc, init, label=" " + mode, **kw)
        worst = w[0] if worst is None else worst
        loss_tol = 10 * kw["tol"]
        for t, (a, b) in enumerate(zip(hl, ol)):
            assert (a is None) == (b is None), f"loss availability differs at t={t}"
            if a is not None:
                assert abs(a - b) <= max(loss_tol * abs(b), 1e-5), f"loss at t={t} ({mode} oracle): {a} vs {b}"
    return worst


def test_tiny_mlp_every_step_fp32():
    _compare(tiny_mlp(K=3, W=2, B=4), seed=1, T=12, every_step=True, tiny=True)


def test_tiny_cnn_every_step_fp32():
    _compare(tiny_cnn(K=2, W=2, B=4), seed=2, T=8, every_step=True, tiny=True)


def test_tiny_resnet_every_step_fp32():
    _compare(tiny_resnet(K=3, W=2, B=4), seed=3, T=10, every_step=True, tiny=True)


def test_tiny_resnet_single_module_is_plain_sgd_fp32():
    _compare(tiny_resnet(K=1, W=1, B=6), seed=4, T=5, every_step=True, tiny=True)


def test_tiny_resnet_bf16():
    _compare(tiny_resnet(K=3, W=2, B=16, precision="bf16"), seed=5, T=10, every_step=True)


def test_tiny_cnn_bf16():
    _compare(tiny_cnn(K=2, W=2, B=16, precision="bf16"), seed=6, T=8, every_step=True)


def test_custom_delays_and_step_size_schedule():
    wl = tiny_mlp(K=3, W=2, B=4)
    _compare(wl, seed=7, T=14, delays=[4, 2, 0], every_step=True,
             lr_schedule=lambda t: 0.05 if t < 8 else 0.005, tiny=True)


def test_cfg0_mlp_full_size_20_steps():
    wl = workload("cfg0_mlp")
    _compare(wl, seed=0, T=wl.steps, every_step=True, tiny=True)


def test_cfg1_cnn_reduced_batch():
    # same K / W / delay structure and layer shapes, B=8 per replica so the oracle leg takes seconds;
    # several M tiles (4*8*32*32 = 8192 rows) and ragged tails in the later layers
    wl = workload("cfg1_cnn", B=8)
    _compare(wl, seed=0, T=2 * (wl.K - 1) + 10)


def test_cfg2_resnet18_reduced_batch_bf16():
    wl = workload("cfg2_resnet18", B=4)
    _compare(wl, seed=0, T=2 * (wl.K - 1) + 10)


def test_cfg2_resnet18_reduced_batch_fp32_arithmetic():
    wl = workload("cfg2_resnet18", B=3, precision="f32")
    _compare(wl, seed=1, T=2 * (wl.K - 1) + 4)


def test_cfg3_resnet56_reduced_batch_bf16():
    # K=8 modules, W=8 replicas, narrow channels (16/32/64): the generic implicit-GEMM path and ring
    # depths up to 15; per-replica batch 2 keeps the oracle leg short
    wl = workload("cfg3_resnet56", B=2)
    _compare(wl, seed=0, T=2 * (wl.K - 1) + 6)


def test_sixteen_channel_layers_bf16():
    # 16 x 16 images, 16 channels: the first block runs on the narrow-layer kernels (direct 16-channel forward /
    # dgrad with sign plane, residual and shortcut-gradient epilogues; 16-channel weight gradient); W = 3 data-groups
    # and batch 5 leave ragged workgroups
    _compare(tiny_resnet(K=2, W=3, B=5, hw=16, c=16, precision="bf16"), seed=8, T=8, every_step=True)
    _compare(tiny_resnet(K=1, W=1, B=1, hw=16, c=16, precision="bf16"), seed=9, T=3, every_step=True)
    # 32 x 32 images (two 16-pixel runs per image row); the second and third block are 32 channels wide at 16 x 16
    _compare(tiny_resnet(K=3, W=2, B=3, hw=32, c=16, precision="bf16"), seed=10, T=8)


def test_uneven_channel_widths_large_pixel_tiles_bf16():
    # 32 -> 128 and 128 -> 64 channels at 65536 pixels: the 256-pixel tiles with one 64-byte channel chunk and
    # 128 output columns (forward of the first), and with several chunks and 64 output columns (its dgrad, and
    # the forward of the second), which the ResNet shapes never select
    _compare(uneven_cnn(), seed=11, T=2)


def test_odd_shapes_fp32_and_bf16():
    # 7 x 9 images, batch 3, stride-2 projection block (parity classes of unequal size, shortcut
    # folded into the dgrad), a conv with 10 output channels (padded channel stride)
    _compare(odd_resnet("f32"), seed=5, T=8, every_step=True, tiny=True)
    _compare(odd_resnet("bf16", c=32), seed=6, T=8)
    _compare(odd_resnet("f32", K=1, W=1, B=1), seed=7, T=4, every_step=True, tiny=True)


def test_repeatable_and_independent_of_stream_layout():
    """The same inputs give bit-identical parameters on a second run (fixed-order reductions, no
    atomics), and also when the modules are serialised on the caller's stream while profiling."""
    import numpy as np
    import torch
    import paper_2509_05679_amd as P
    from dds_inputs import make_batch, make_params
    wl = workload("cfg2_resnet18", B=4)

    def run(profile_mode):
        tr = P.Trainer(P.Spec.from_workload(wl), wl.W)
        init = make_params(wl, 0)
        for k0 in range(wl.K):
            tr.dds_set_params(k0, init[k0])
        if profile_mode:
            tr.dds_profile(profile_mode)
        for t in range(2 * (wl.K - 1) + 4):
            xs = [torch.from_numpy(make_batch(wl, 0, t, s)[0]).cuda() for s in range(wl.W)]
            ys = [torch.from_numpy(make_batch(wl, 0, t, s)[1]).cuda() for s in range(wl.W)]
            tr.dds_step(xs, ys)
        torch.cuda.synchronize()
        out = [tr.dds_get_params(k0) for k0 in range(wl.K)]
        tr.close()
        return out

    a, b, c = run(0), run(0), run(2)
    for k0 in range(wl.K):
        assert np.array_equal(a[k0], b[k0]), f"module {k0}: two identical runs differ"
        assert np.array_equal(a[k0], c[k0]), f"module {k0}: serialised run differs from the concurrent one"


def test_paper_resnet20_shapes_reduced_batch_bf16():
    # The paper's own experiment shapes (Section 5): ResNet-20, S = 4 data-groups, K = 2 modules and
    # the centralised K = 1 special case; per-group batch 7 (odd, like the paper's 194: ragged tiles).
    wl = workload("paper_r20_S4K2", B=7)
    _compare(wl, seed=2, T=wl.steps)
    wl = workload("paper_r20_S1K1", B=7)
    _compare(wl, seed=3, T=6)


def test_cfg4_resnet34w_reduced_batch_bf16():
    wl = workload("cfg4_resnet34w", B=1, W=4)
    _compare(wl, seed=0, T=2 * (wl.K - 1) + 3)
