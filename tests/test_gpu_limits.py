"""GPU tests at the edges of what the library accepts: the largest replica count, a long module
chain with one-sample mini-batches, and the error paths of calls that need a context."""
import math

import numpy as np
import pytest

from dds_inputs import make_batch, make_params
from dds_inputs.configs import tiny_mlp, tiny_resnet
from parity import check_parity, flat_init, run_hip, run_oracle, thresholds

pytestmark = pytest.mark.gpu


def _check(wl, seed, T, **kw):
    hip, hl = run_hip(wl, seed, T, every_step=True, **kw)
    orc, ol = run_oracle(wl, seed, T, every_step=True, **kw)
    init = flat_init(wl, seed)
    (_, th), = thresholds("f32", tiny=True)
    check_parity(wl, hip, orc, init, label=" limits", **th)
    for a, b in zip(hl, ol):
        assert (a is None) == (b is None)
        if a is not None:
            assert abs(a - b) <= 1e-3 * abs(b) + 1e-6


def test_thirty_two_data_groups_of_one_sample():
    # W = 32 is the largest replica count dds_create accepts; B = 1: every mean is over one sample
    _check(tiny_mlp(K=3, W=32, B=1), seed=31, T=8)


def test_eight_modules_deep_chain_one_sample_batches():
    # K = 8: ring depths 15, 13, ..., 1; the first module updates for the first time at iteration 14
    _check(tiny_mlp(K=8, W=1, B=1), seed=32, T=20)


def test_longest_allowed_delays_on_a_short_chain():
    # delays far beyond the paper's d_k = K-1-k: ring depth 2*9+1 = 19 for module 0
    _check(tiny_resnet(K=2, W=2, B=2), seed=33, T=24, delays=[9, 3])


def test_error_paths_of_context_calls():
    import torch
    import paper_2509_05679_amd as P
    wl = tiny_resnet(K=2, W=2, B=2)
    tr = P.Trainer(P.Spec.from_workload(wl), wl.W)
    init = make_params(wl, 0)
    lib, ctx = P.lib, tr.ctx
    n0 = tr.dds_param_count(0)
    buf = torch.zeros(n0 + 1, dtype=torch.float32, device="cuda")
    stream = tr._stream()
    # wrong element count, bad module, null pointer
    assert lib.dds_set_params(ctx, 0, buf.data_ptr(), n0 + 1, stream) == P.DDS_EINVAL
    assert lib.dds_get_params(ctx, 5, buf.data_ptr(), n0, stream) == P.DDS_EINVAL
    assert lib.dds_get_params(ctx, 0, None, n0, stream) == P.DDS_EINVAL
    assert lib.dds_get_params_replica(ctx, 0, 2, buf.data_ptr(), n0, stream) == P.DDS_EINVAL
    assert lib.dds_param_count(ctx, -1) == P.DDS_EINVAL
    # no loss before the last module has forwarded anything
    with pytest.raises(P.DdsError) as e:
        tr.dds_get_loss()
    assert e.value.code == P.DDS_EINVAL and "loss" in str(e.value)
    for k0 in range(wl.K):
        tr.dds_set_params(k0, init[k0])
    xs = [torch.from_numpy(make_batch(wl, 0, 0, s)[0]).cuda() for s in range(wl.W)]
    ys = [torch.from_numpy(make_batch(wl, 0, 0, s)[1]).cuda() for s in range(wl.W)]
    # a null batch pointer is refused before anything is enqueued
    import ctypes as C
    xp = (C.c_void_p * 2)(xs[0].data_ptr(), None)
    yp = (C.c_void_p * 2)(ys[0].data_ptr(), ys[1].data_ptr())
    assert lib.dds_step(ctx, xp, yp, math.nan, stream) == P.DDS_EINVAL
    assert tr.dds_step_count() == 0
    tr.dds_step(xs, ys)
    assert tr.dds_step_count() == 1
    # weights can only be set before the first step
    flat = np.concatenate([p.ravel() for p in init[0]])
    dev = torch.from_numpy(flat).cuda()
    assert lib.dds_set_params(ctx, 0, dev.data_ptr(), flat.size, stream) == P.DDS_EINVAL
    # without a mixing matrix every data-group holds the same weights and the disagreement is exactly 0
    torch.cuda.synchronize()
    assert np.array_equal(tr.dds_get_params(1), tr.dds_get_params_replica(1, 1))
    assert tr.dds_consensus_error() == 0.0
    tr.close()
    # an arena that is too small is refused
    spec = P.Spec.from_workload(wl)
    need = P.dds_arena_bytes(spec, wl.K, wl.W)
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    out = C.c_void_p()
    base = (arena.data_ptr() + 255) // 256 * 256
    assert lib.dds_create(C.byref(spec.c), wl.K, wl.W, None, base, need // 2, C.byref(out)) == P.DDS_ENOMEM


@pytest.mark.parametrize("name,B,steps", [("cfg2_resnet18", 16, 40), ("cfg3_resnet56", 4, 40), ("cfg1_cnn", 16, 30)])
def test_run_ahead_across_iterations_is_bit_identical_to_serial_execution(name, B, steps):
    """With three or more modules a module program starts as soon as its neighbours' previous iteration is
    done, i.e. before the other modules have finished the current one. Batches are resident and the steps are
    enqueued back to back so that the programs really overlap across iterations; the result must equal, bit
    for bit, the run in which the modules execute one after another on the caller's stream."""
    import torch
    import paper_2509_05679_amd as P
    from dds_inputs import workload
    wl = workload(name, B=B)
    init = make_params(wl, 7)
    pool = 5
    xs = [[torch.from_numpy(make_batch(wl, 7, t, s)[0]).cuda() for s in range(wl.W)] for t in range(pool)]
    ys = [[torch.from_numpy(make_batch(wl, 7, t, s)[1]).cuda() for s in range(wl.W)] for t in range(pool)]

    def run(mode):
        tr = P.Trainer(P.Spec.from_workload(wl), wl.W)
        for k0 in range(wl.K):
            tr.dds_set_params(k0, init[k0])
        if mode:
            tr.dds_profile(mode)
        for t in range(steps):
            tr.dds_step(xs[t % pool], ys[t % pool])
        torch.cuda.synchronize()
        out = [tr.dds_get_params(k0) for k0 in range(wl.K)]
        tr.close()
        return out

    ahead, serial = run(0), run(2)
    for k0 in range(wl.K):
        assert np.isfinite(ahead[k0]).all()
        assert np.array_equal(ahead[k0], serial[k0]), f"module {k0}"


def test_switching_the_callers_stream_between_iterations():
    """Module 0 runs on the caller's stream: when the caller passes another stream the library orders the new
    iteration after the previous one itself. Alternating between two streams must not change a bit."""
    import ctypes as C
    import torch
    import paper_2509_05679_amd as P
    from dds_inputs import workload
    wl = workload("cfg2_resnet18", B=8)
    init = make_params(wl, 9)
    xs = [torch.from_numpy(make_batch(wl, 9, 0, s)[0]).cuda() for s in range(wl.W)]
    ys = [torch.from_numpy(make_batch(wl, 9, 0, s)[1]).cuda() for s in range(wl.W)]
    side = torch.cuda.Stream()  # default priority
    torch.cuda.synchronize()

    def run(alternate):
        tr = P.Trainer(P.Spec.from_workload(wl), wl.W)
        for k0 in range(wl.K):
            tr.dds_set_params(k0, init[k0])
        torch.cuda.synchronize()
        for t in range(16):
            if alternate and t % 2:
                with torch.cuda.stream(side):
                    tr.dds_step(xs, ys)
            else:
                tr.dds_step(xs, ys)
        torch.cuda.synchronize()
        out = [tr.dds_get_params(k0) for k0 in range(wl.K)]
        tr.close()
        return out

    same, alt = run(False), run(True)
    for k0 in range(wl.K):
        assert np.array_equal(same[k0], alt[k0]), f"module {k0}"
