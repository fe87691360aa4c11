"""GPU parity of the general mixing step (Section 2.3 / 3.3: a communication graph with matrix P,
every data-group keeping its own weights) against the CPU oracle, data-group by data-group,
and of the disagreement measure delta(t) of the experiment section."""
import numpy as np
import pytest

from dds_inputs import make_batch, make_params, workload
from dds_inputs.configs import complete_mixing, ring_mixing, tiny_cnn, tiny_mlp, tiny_resnet
from parity import bf16_round, check_parity, flat_init, thresholds

pytestmark = pytest.mark.gpu


def _run_hip(wl, seed, T, mixing, delays=None):
    import torch
    import paper_2509_05679_amd as P
    tr = P.Trainer(P.Spec.from_workload(wl, mixing), wl.W, delays)
    init = make_params(wl, seed)
    for k0 in range(wl.K):
        tr.dds_set_params(k0, init[k0])
    traj, deltas = [], []
    for t in range(T):
        xs, ys = [], []
        for s in range(wl.W):
            x, y = make_batch(wl, seed, t, s)
            xs.append(torch.from_numpy(x).cuda())
            ys.append(torch.from_numpy(y).cuda())
        tr.dds_step(xs, ys)
        torch.cuda.synchronize()
        traj.append([[tr.dds_get_params_replica(k0, s) for k0 in range(wl.K)] for s in range(wl.W)])
        deltas.append(tr.dds_consensus_error())
    tr.close()
    return traj, deltas


def _run_oracle(wl, seed, T, mixing, delays=None, q=None):
    import torch
    from oracle import fdg
    Pm = None if mixing is None else torch.tensor(mixing, dtype=torch.float64)
    pipe = fdg.Pipeline(wl.ops, wl.bounds, wl.W, make_params(wl, seed), wl.lr, wl.momentum, delays, Pm, q=q)
    pipe.keep_history = False
    traj, deltas = [], []
    for t in range(T):
        pipe.step([make_batch(wl, seed, t, s) for s in range(wl.W)])
        traj.append([[np.concatenate([p.numpy().ravel() for p in pipe.w[s][k0]]) for k0 in range(wl.K)]
                     for s in range(wl.W)])
        deltas.append(fdg.consensus_error(pipe.w))
    return traj, deltas


def _compare(wl, seed, T, mixing, delays=None, delta_rel=None, tiny=True):
    delta_rel = (1e-3 if wl.precision == "f32" else 1e-1) if delta_rel is None else delta_rel
    print(f"[gossip] {wl.name} K={wl.K} W={wl.W} B={wl.B} {wl.precision} mu={wl.momentum} T={T} seed={seed}", flush=True)
    hip, hd = _run_hip(wl, seed, T, mixing, delays)
    init = flat_init(wl, seed)
    od_exact = None
    for mode, kw in thresholds(wl.precision, tiny):
        orc, od = _run_oracle(wl, seed, T, mixing, delays, q=bf16_round() if mode == "rounded" else None)
        for s in range(wl.W):  # every data-group's own weights, after every iteration
            check_parity(wl, [hip[t][s] for t in range(T)], [orc[t][s] for t in range(T)], init,
                         label=f" gossip {mode} group {s}", verbose=(s == 0), **kw)
        if mode == "exact":
            od_exact = od
            for t in range(T):
                assert abs(hd[t] - od[t]) <= delta_rel * od[t] + 1e-7, f"delta({t}): hip {hd[t]:.6e} oracle {od[t]:.6e}"
    print(f"[gossip] delta(T-1) hip {hd[-1]:.4e} oracle {od_exact[-1]:.4e}", flush=True)
    return hd, od_exact


def test_ring_of_four_tiny_resnet_fp32():
    wl = tiny_resnet(K=3, W=4, B=4)
    hd, od = _compare(wl, seed=11, T=10, mixing=ring_mixing(4, 0.3))
    assert od[-1] > 1e-6, "the data-groups must actually disagree for this test to say anything"


def test_ring_of_three_with_momentum_and_custom_delays_fp32():
    wl = tiny_cnn(K=2, W=3, B=4, momentum=0.9)
    _compare(wl, seed=12, T=9, mixing=ring_mixing(3, 0.25), delays=[2, 0])


def test_single_edge_mlp_fp32():
    _compare(tiny_mlp(K=3, W=2, B=4), seed=13, T=12, mixing=ring_mixing(2, 0.4))


def test_isolated_data_groups_identity_matrix_fp32():
    # P = I: no communication at all, every data-group runs the decoupled recurrence alone
    wl = tiny_resnet(K=2, W=3, B=4)
    eye = [[1.0 if i == j else 0.0 for j in range(3)] for i in range(3)]
    _compare(wl, seed=14, T=8, mixing=eye)


def test_ring_of_four_sixteen_channel_layers_bf16():
    # the narrow-layer kernels with every data-group's own weights in one launch (weights picked per wave)
    wl = tiny_resnet(K=2, W=4, B=4, hw=16, c=16, precision="bf16")
    _compare(wl, seed=18, T=8, mixing=ring_mixing(4, 0.3), tiny=False)


def test_complete_graph_reproduces_exact_mean_path():
    """P = (1/W) 11^T through the per-data-group code must land on the single-copy hot path."""
    import torch
    import paper_2509_05679_amd as P
    wl = tiny_resnet(K=3, W=4, B=4)
    T, seed = 10, 15
    hip, hd = _run_hip(wl, seed, T, complete_mixing(4))
    tr = P.Trainer(P.Spec.from_workload(wl), wl.W)
    init = make_params(wl, seed)
    for k0 in range(wl.K):
        tr.dds_set_params(k0, init[k0])
    for t in range(T):
        xs, ys = zip(*[make_batch(wl, seed, t, s) for s in range(wl.W)])
        tr.dds_step([torch.from_numpy(x).cuda() for x in xs], [torch.from_numpy(y).cuda() for y in ys])
    torch.cuda.synchronize()
    assert tr.dds_consensus_error() == 0.0
    for k0 in range(wl.K):
        ref = tr.dds_get_params(k0)
        np.testing.assert_array_equal(ref, tr.dds_get_params_replica(k0, wl.W - 1))
        for s in range(wl.W):
            err = np.linalg.norm(hip[-1][s][k0].astype(np.float64) - ref) / np.linalg.norm(ref)
            assert err < 2e-6, f"module {k0} data-group {s}: {err:.3e}"
    tr.close()
    assert max(hd) < 1e-5


def test_ring_of_four_resnet18_shapes_bf16():
    # the MFMA kernels launched once per data-group (4 images each) with that group's own weights and snapshots
    wl = workload("cfg2_resnet18", B=4)
    _compare(wl, seed=16, T=2 * (wl.K - 1) + 6, mixing=ring_mixing(4, 0.3), tiny=False)


def test_ring_of_four_cnn_shapes_fp32():
    # fp32 arithmetic at the CNN configuration's layer shapes (64-512 channels, max-pooling, momentum 0.9):
    # the fp32 asynchronous kernels with one launch per layer for the four data-groups' own weights
    wl = workload("cfg1_cnn", B=8)
    _compare(wl, seed=17, T=2 * (wl.K - 1) + 6, mixing=ring_mixing(4, 0.3), tiny=False)
