"""Bit-exact checks, on the device, of delay-buffer indexing and mini-batch assignment (Section 3.2:
module k forwards mini-batch t-k+1 and back-propagates mini-batch t-2K+k+1 with the weights of iteration
t-2K+2k; zero-based here: f = t-k0, b = t-k0-2d, weights of t-2d).

Tag test. A chain of K identity modules (linear 16 -> 16 with the identity matrix and zero bias, ReLU; the last
one feeds softmax cross-entropy) run with step size 0 moves every mini-batch through the pipeline unchanged,
in exact fp32 arithmetic: inputs are positive integers that encode (iteration, data-group, sample, feature), one
feature per sample is raised by 512 so that the softmax is exactly one-hot, hence the loss gradient of a sample
is exactly +1/B at that feature and -1/B at its label, and it too travels back through the identity modules
unchanged. After every iteration EVERY slot of every activation ring, error mailbox and the label queue is read
back (dds_debug_read) and compared, byte for byte, with the content the oracle's schedule integers say it must
hold. A final iteration with step size 1 then makes the pairing inside the backward pass observable: the updated
weights I - (1/W) sum_s dY_s^T X_s are exact small dyadic numbers that name which mini-batch's activations met
which mini-batch's error gradient in every module.

Snapshot test. On a small fp32 network that really trains, every slot of every weight-snapshot ring must hold,
bit for bit, the transposed master weights of the iteration the schedule assigns to it (dds_get_params history)."""
import numpy as np
import pytest

from dds_inputs.configs import Workload, _linear, _relu, tiny_mlp
from dds_inputs import make_batch, make_params
from oracle import fdg

pytestmark = pytest.mark.gpu

C = 16  # features = classes


def _chain(K, W, B):
    ops, bounds = [], [0]
    for k0 in range(K):
        ops += [_linear(C, C), _relu()] if k0 < K - 1 else [_linear(C, C), {"op": "softmax_ce"}]
        bounds.append(len(ops))
    return Workload(name=f"identity_chain_K{K}", ops=ops, bounds=bounds, K=K, W=W, B=B, in_shape=(C, 1, 1), classes=C,
                    precision="f32", lr=0.0, momentum=0.0, steps=0)


def _ident(t, s, n, W, B):
    return n + B * (s + W * t)


def _tags(t, W, B):
    """Mini-batch sampled at iteration t: x [W][B, C] (positive integers), labels [W][B], and the exact loss
    gradient rows [W][B, C] of a softmax that is one-hot at the raised feature."""
    xs, ys, gs = [], [], []
    for s in range(W):
        x = np.zeros((B, C), dtype=np.float32)
        y = np.zeros((B,), dtype=np.int32)
        g = np.zeros((B, C), dtype=np.float32)
        for n in range(B):
            i = _ident(t, s, n, W, B)
            a = (7 * i + 3) % C
            lab = (a + 1 + (i // C) % (C - 1)) % C
            x[n] = 1024 * i + 1 + np.arange(C)
            x[n, a] += 512
            y[n] = lab
            g[n, a] += 1.0 / B
            g[n, lab] -= 1.0 / B
        xs.append(x), ys.append(y), gs.append(g)
    return xs, ys, gs


def _run_tag_test(K, delays, W, B, t_final):
    import torch
    import paper_2509_05679_amd as P
    wl = _chain(K, W, B)
    d = fdg.paper_delays(K) if delays is None else delays
    tr = P.Trainer(P.Spec.from_workload(wl), W, delays)
    eye = [np.eye(C, dtype=np.float32), np.zeros(C, dtype=np.float32)]
    for k0 in range(K):
        tr.dds_set_params(k0, eye)
    R = [2 * d[k0] + 1 for k0 in range(K)]
    err_depth = [2 * (d[k0] - d[k0 + 1]) for k0 in range(K - 1)]
    depth = K + 2 * d[K - 1]
    # what each slot must hold: a mini-batch id, or None (never written: the arena starts zeroed)
    ring_in = [None] * R[0]
    ring_out = [[None] * R[k0] for k0 in range(K)]
    err = [[None] * n for n in err_depth]
    labels = [None] * depth
    cat = lambda rows: np.concatenate(rows, axis=0)  # data-groups are stacked along the sample axis

    def expect(batch, what):
        if batch is None:
            return np.zeros((W * B, 1), dtype=np.int32) if what == "y" else np.zeros((W * B, C), dtype=np.float32)
        xs, ys, gs = _tags(batch, W, B)
        return {"x": cat(xs), "y": cat(ys).reshape(-1, 1), "g": cat(gs)}[what]

    for t in range(t_final + 1):
        last_step = t == t_final
        xs, ys, _ = _tags(t, W, B)
        tr.dds_step([torch.from_numpy(x.reshape(B, C, 1, 1)).cuda() for x in xs],
                    [torch.from_numpy(y).cuda() for y in ys], 1.0 if last_step else 0.0)
        sch = fdg.schedule(t, K, delays)
        labels[sch[0]["label_write"]] = t
        ring_in[sch[0]["fwd_slot"]] = t
        for rec in sch:
            k0 = rec["k0"]
            if rec["f"] >= 0:
                ring_out[k0][rec["fwd_slot"]] = rec["f"]
            if rec["b"] >= 0 and k0 > 0:
                err[k0 - 1][rec["err_write"]] = rec["b"]
        # every slot of every delay buffer, byte for byte
        for j in range(R[0]):
            got = tr.dds_debug_read(P.DDS_DBG_INPUT, 0, j).view(np.float32).reshape(W * B, C)
            assert np.array_equal(got, expect(ring_in[j], "x")), ("input ring", t, j)
        for k0 in range(K):
            for j in range(R[k0]):
                got = tr.dds_debug_read(P.DDS_DBG_OUTPUT, k0, j).view(np.float32).reshape(W * B, C)
                assert np.array_equal(got, expect(ring_out[k0][j], "x")), ("output ring", t, k0, j)
        for k0 in range(K - 1):
            for j in range(err_depth[k0]):
                got = tr.dds_debug_read(P.DDS_DBG_ERROR, k0, j).view(np.float32).reshape(W * B, C)
                assert np.array_equal(got, expect(err[k0][j], "g")), ("error mailbox", t, k0, j)
        for j in range(depth):
            got = tr.dds_debug_read(P.DDS_DBG_LABELS, 0, j).view(np.int32).reshape(W * B, 1)
            assert np.array_equal(got, expect(labels[j], "y")), ("label queue", t, j)
        if not last_step:
            for k0 in range(K):  # step size 0: the identity stays the identity
                assert np.array_equal(tr.dds_get_params(k0), np.concatenate([eye[0].ravel(), eye[1]])), (t, k0)
    # the final iteration used step size 1: which activations met which error gradient, module by module
    sch = fdg.schedule(t_final, K, delays)
    for rec in sch:
        k0 = rec["k0"]
        Wm, bias = np.eye(C, dtype=np.float64), np.zeros(C, dtype=np.float64)
        if rec["b"] >= 0:
            xs, _, gs = _tags(rec["b"], W, B)
            for s in range(W):
                Wm -= gs[s].astype(np.float64).T @ xs[s].astype(np.float64) / W
                bias -= gs[s].astype(np.float64).sum(axis=0) / W
        want = np.concatenate([Wm.ravel(), bias]).astype(np.float32)
        assert np.array_equal(want.astype(np.float64), np.concatenate([Wm.ravel(), bias])), "expected values are exact in fp32"
        got = tr.dds_get_params(k0)
        assert np.array_equal(got, want), ("pairing inside the backward pass", t_final, k0, rec["b"])
    tr.close()


@pytest.mark.parametrize("K,delays", [(3, None), (8, None), (3, [4, 2, 0]), (2, [3, 1]), (1, None)])
def test_tagged_mini_batches_land_in_the_slots_the_schedule_names(K, delays):
    d = fdg.paper_delays(K) if delays is None else delays
    # final iterations: the first one where every module back-propagates, one a few later, one after module 0's
    # ring has wrapped around
    first_full = max(k0 + 2 * d[k0] for k0 in range(K))
    for t_final in (first_full, first_full + 3, first_full + 2 * d[0] + 2):
        print(f"[tags] K={K} delays={delays} final iteration {t_final}", flush=True)
        _run_tag_test(K, delays, W=2, B=4, t_final=t_final)


def test_partially_filled_pipeline_updates_only_modules_with_a_gradient():
    # final iteration before module 0 has a gradient: its weights must stay the identity exactly
    _run_tag_test(3, None, W=2, B=4, t_final=2)


@pytest.mark.parametrize("K,delays", [(3, None), (3, [4, 2, 0])])
def test_snapshot_ring_slots_hold_the_weights_of_the_scheduled_iteration(K, delays):
    import torch
    import paper_2509_05679_amd as P
    wl = tiny_mlp(K=K, W=2, B=4)
    d = fdg.paper_delays(K) if delays is None else delays
    seed = 51
    tr = P.Trainer(P.Spec.from_workload(wl), wl.W, delays)
    init = make_params(wl, seed)
    for k0 in range(K):
        tr.dds_set_params(k0, init[k0])
    versions = [[tr.dds_get_params(k0)] for k0 in range(K)]     # versions[k0][v] = weights at the start of iteration v
    held = [[0] * (2 * d[k0] + 1) for k0 in range(K)]           # version each snapshot slot holds
    cin = [wl.ops[wl.bounds[k0]]["cin"] for k0 in range(K)]
    cout = [wl.ops[wl.bounds[k0]]["cout"] for k0 in range(K)]
    for t in range(2 * (K - 1) + 2 * d[0] + 6):
        xs, ys = zip(*[make_batch(wl, seed, t, s) for s in range(wl.W)])
        tr.dds_step([torch.from_numpy(x).cuda() for x in xs], [torch.from_numpy(y).cuda() for y in ys])
        sch = fdg.schedule(t, K, delays)
        for rec in sch:
            k0 = rec["k0"]
            versions[k0].append(tr.dds_get_params(k0))
            if rec["b"] >= 0:
                # what this iteration's backward read: the slot must hold the weights of iteration t - 2d (an
                # earlier version number with the same content while no update had happened yet)
                assert np.array_equal(versions[k0][held[k0][rec["bwd_slot"]]], versions[k0][t - 2 * d[k0]]), (t, k0)
                held[k0][rec["snap_write"]] = t + 1
            else:
                assert np.array_equal(versions[k0][-1], versions[k0][0]), (t, k0)
        for k0 in range(1, K):  # module 0's only layer has nothing to back-propagate into: no snapshots
            cpad = (cout[k0] + 3) // 4 * 4
            for j in range(2 * d[k0] + 1):
                got = tr.dds_debug_read(P.DDS_DBG_SNAPSHOT, k0, j, index=0).view(np.float32).reshape(cin[k0], cpad)
                w = versions[k0][held[k0][j]][:cout[k0] * cin[k0]].reshape(cout[k0], cin[k0])
                want = np.zeros((cin[k0], cpad), dtype=np.float32)
                want[:, :cout[k0]] = w.T
                assert np.array_equal(got, want), ("snapshot ring", t, k0, j, held[k0][j])
        with pytest.raises(P.DdsError):
            tr.dds_debug_read(P.DDS_DBG_SNAPSHOT, 0, 0, index=0)
    assert all(len(set(map(bytes, v))) > 3 for v in versions), "the weights must actually change for this test to say anything"
    tr.close()
