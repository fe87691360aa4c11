"""Pins for the oracle's training recurrence (schedule, stale weights, replica
mean, reductions to plain SGD, consensus)."""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from dds_inputs import make_batch, make_params
from dds_inputs.configs import tiny_cnn, tiny_mlp, tiny_resnet
from oracle import fdg, network as N

DT = torch.float64
GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ schedule
def test_schedule_matches_paper_table_for_three_modules():
    rows = [l.split() for l in open(os.path.join(GOLD, "fdg_schedule_K3.txt")) if not l.startswith("#")]
    for t, k, f, b, wv in (map(int, r) for r in rows):
        rec = fdg.schedule(t, 3)[k - 1]
        assert (rec["f"] if rec["f"] >= 0 else -1) == f
        assert (rec["b"] if rec["b"] >= 0 else -1) == b
        if b >= 0:
            # the backward uses the weights the module held when it forwarded batch b
            assert b + (k - 1) == wv


def _simulate_hops(K, d, T):
    """Event simulation, independent of the closed forms: a batch moves one module
    down per iteration; module k0 back-propagates a batch once it holds the error
    gradient for it (posted by module k0+1 in an EARLIER iteration) and its own
    configured wait of 2*d[k0] iterations since the forward has elapsed."""
    fwd_at = {}
    bwd_at = {}
    for t in range(T):
        for k0 in range(K):
            tau = t - k0  # batch arriving now: sampled at tau, one hop per iteration
            if tau >= 0:
                fwd_at[(k0, tau)] = t
        for k0 in range(K - 1, -1, -1):
            for tau in range(t + 1):
                if (k0, tau) in bwd_at or (k0, tau) not in fwd_at:
                    continue
                if t - fwd_at[(k0, tau)] < 2 * d[k0]:
                    continue
                if k0 < K - 1 and not ((k0 + 1, tau) in bwd_at and bwd_at[(k0 + 1, tau)] < t):
                    raise AssertionError("error gradient not available in time")
                bwd_at[(k0, tau)] = t
    return fwd_at, bwd_at


@pytest.mark.parametrize("K", range(1, 9))
def test_schedule_closed_forms_against_hop_simulation(K):
    T = 64
    d = fdg.paper_delays(K)
    fwd_at, bwd_at = _simulate_hops(K, d, T)
    for t in range(T):
        for rec in fdg.schedule(t, K):
            k0 = rec["k0"]
            if rec["f"] >= 0:
                assert fwd_at[(k0, rec["f"])] == t
            else:
                assert all(v != t for (kk, _), v in fwd_at.items() if kk == k0)
            if rec["b"] >= 0:
                assert bwd_at[(k0, rec["b"])] == t
                # paper: batch t-2K+k+1 with 1-based k
                assert rec["b"] == t - 2 * K + (k0 + 1) + 1
            else:
                assert all(v != t for (kk, _), v in bwd_at.items() if kk == k0)


@pytest.mark.parametrize("K,d", [(3, [4, 2, 0]), (3, [3, 1, 0]), (4, [5, 4, 2, 1]), (2, [1, 0]), (2, [3, 1])])
def test_ring_and_mailbox_slots_never_clobber_live_data(K, d):
    """Brute-force the slot arithmetic: write tags into rings of the advertised depth
    and check every read returns the batch the closed form names."""
    fdg.check_delays(K, d)
    rings = [dict() for _ in range(K)]
    errs = [dict() for _ in range(K)]
    labels = {}
    snaps = [{j: 0 for j in range(2 * d[k0] + 1)} for k0 in range(K)]  # every slot starts with the initial weights w(0)
    for t in range(80):
        sch = fdg.schedule(t, K, d)
        labels[sch[0]["label_write"]] = t
        # reads happen against the state left by earlier iterations (plus own forward)
        for rec in sch:
            k0 = rec["k0"]
            if rec["f"] >= 0:
                if k0 > 0:  # the input is still in the ring of the module below
                    assert rings[k0 - 1][rec["in_fwd_slot"]] == rec["f"]
                rings[k0][rec["fwd_slot"]] = rec["f"]
            if k0 == K - 1 and rec["f"] >= 0:
                assert labels[rec["label_slot"]] == rec["f"]
            if k0 == K - 1 and rec["b"] >= 0:
                assert labels[rec["label_bwd_slot"]] == rec["b"]
            if rec["b"] >= 0:
                # the snapshot in the backward slot is the weight version the forward of batch b used:
                # w(b + k0) = w(t - 2 d), Section 3.2's w(t - 2K + 2k) under the paper's delays
                assert snaps[k0][rec["bwd_slot"]] == rec["b"] + k0 == t - 2 * d[k0]
        pending = []
        for rec in sch:
            k0 = rec["k0"]
            if rec["b"] >= 0:
                assert rings[k0][rec["bwd_slot"]] == rec["b"]
                if k0 < K - 1:
                    assert errs[k0][rec["err_read"]] == rec["b"]
                if k0 > 0:
                    pending.append((k0 - 1, rec["err_write"], rec["b"]))
                # the module below reads this module's input from the ring of k0-1
                if k0 > 0:
                    assert rings[k0 - 1][rec["in_bwd_slot"]] == rec["b"]
        for k0, slot, b in pending:
            errs[k0][slot] = b
        for rec in sch:  # weights after this iteration = version t+1
            snaps[rec["k0"]][rec["snap_write"]] = t + 1


def test_delay_causality_is_enforced():
    with pytest.raises(ValueError):
        fdg.check_delays(3, [1, 1, 0])
    with pytest.raises(ValueError):
        fdg.check_delays(2, [0, 0])
    fdg.check_delays(1, [0])
    fdg.check_delays(4, [3, 2, 1, 0])


# ------------------------------------------------------------------ recurrence
def _run(wl, seed=0, T=None, P=None, delays=None, S=None, init=None):
    S = wl.W if S is None else S
    pipe = fdg.Pipeline(wl.ops, wl.bounds, S, make_params(wl, seed) if init is None else init,
                        wl.lr, wl.momentum, delays, P)
    losses = []
    for t in range(wl.steps if T is None else T):
        losses.append(pipe.step([make_batch(wl, seed, t, s) for s in range(S)]))
    return pipe, losses


def _plain_sgd(wl, seed, T, concat_replicas):
    """Textbook mini-batch SGD (Section 2.1) with torch autograd, written separately."""
    ps = [torch.as_tensor(p, dtype=DT).clone().requires_grad_() for m in make_params(wl, seed) for p in m]
    vel = [torch.zeros_like(p) for p in ps]
    slots = N.param_slots(wl.ops)
    for t in range(T):
        xs, ys = zip(*[make_batch(wl, seed, t, s) for s in range(concat_replicas)])
        h = torch.as_tensor(np.concatenate(xs), dtype=DT)
        y = torch.as_tensor(np.concatenate(ys), dtype=torch.int64)
        stack = []
        for op, s in zip(wl.ops, slots):
            k = op["op"]
            if k == "conv":
                h = F.conv2d(h, ps[s], ps[s + 1], stride=op["stride"], padding=op["pad"])
            elif k == "linear":
                h = F.linear(h.flatten(1), ps[s], ps[s + 1]).view(h.shape[0], -1, 1, 1)
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
                sh = F.conv2d(xin, ps[s], ps[s + 1], stride=sc["stride"], padding=sc["pad"]) if sc else xin
                h = sh + op["scale"] * h
            elif k == "softmax_ce":
                h = F.cross_entropy(h.flatten(1), y)
        gs = torch.autograd.grad(h, ps)
        with torch.no_grad():
            for p, v, g in zip(ps, vel, gs):
                v.mul_(wl.momentum).add_(g)
                p.sub_(wl.lr * v)
    return [p.detach() for p in ps]


@pytest.mark.parametrize("make", [tiny_resnet, tiny_cnn])
def test_one_module_one_replica_is_plain_sgd(make):
    wl = make(K=1, W=1)
    pipe, _ = _run(wl, seed=5, T=6)
    ref = _plain_sgd(wl, 5, 6, 1)
    for a, b in zip([p for m in pipe.params() for p in m], ref):
        assert torch.allclose(a, b, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("make", [tiny_resnet, tiny_cnn])
def test_replica_mean_equals_concatenated_batch(make):
    """K=1: W data-groups with exact-mean mixing == plain SGD on the union batch."""
    wl = make(K=1, W=3)
    pipe, _ = _run(wl, seed=6, T=5)
    ref = _plain_sgd(wl, 6, 5, 3)
    for a, b in zip([p for m in pipe.params() for p in m], ref):
        assert torch.allclose(a, b, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("make,K", [(tiny_resnet, 3), (tiny_cnn, 2), (tiny_mlp, 3), (tiny_resnet, 2)])
def test_pipeline_equals_definition_at_skewed_weights(make, K):
    """The pipelined execution (mailboxes, saved activations, weight snapshots) applies
    exactly the gradient of the loss at col{ w_k(tau+k-1) } that the definition names."""
    wl = make(K=K, W=2)
    T = 2 * (K - 1) + 5
    pipe, _ = _run(wl, seed=7, T=T)
    hist = fdg.definition_replay(wl.ops, wl.bounds, wl.W, make_params(wl, 7), wl.lr, wl.momentum,
                                 None, None, lambda b, s: make_batch(wl, 7, b, s), T)
    final = hist[T]
    for s in range(wl.W):
        for k0 in range(K):
            for a, b in zip(pipe.w[s][k0], final[s][k0]):
                assert torch.allclose(a, b, rtol=1e-12, atol=1e-14)
    # a pipeline that back-propagated through its CURRENT weights would differ
    changed = any(not torch.equal(a, b) for a, b in zip(hist[T][0][0], hist[0][0][0]))
    assert changed


def test_pipeline_equals_definition_with_longer_delays():
    wl = tiny_mlp(K=3, W=2)
    d = [4, 2, 0]
    T = 14
    pipe, _ = _run(wl, seed=8, T=T, delays=d)
    hist = fdg.definition_replay(wl.ops, wl.bounds, wl.W, make_params(wl, 8), wl.lr, 0.0, d, None,
                                 lambda b, s: make_batch(wl, 8, b, s), T)
    for k0 in range(3):
        for a, b in zip(pipe.w[0][k0], hist[T][0][k0]):
            assert torch.allclose(a, b, rtol=1e-12, atol=1e-14)


def test_stale_weights_matter():
    """Sanity of the pin above: evaluating the definition at the CURRENT weights of
    every module (no skew) gives a different trajectory, so the test can fail."""
    wl = tiny_mlp(K=3, W=1)
    T = 9
    pipe, _ = _run(wl, seed=9, T=T)
    w = [[torch.as_tensor(p, dtype=DT) for p in m] for m in make_params(wl, 9)]
    for t in range(T):
        new = []
        for k0 in range(3):
            b = t - k0 - 2 * (2 - k0)
            if b < 0:
                new.append(w[k0])
                continue
            x, y = make_batch(wl, 9, b, 0)
            g, _ = fdg.definition_gradient(wl.ops, wl.bounds, w, x, y)
            new.append([p - wl.lr * gi for p, gi in zip(w[k0], g[k0])])
        w = new
    assert not torch.allclose(pipe.w[0][0][0], w[0][0], rtol=1e-6, atol=1e-9)


def test_warmup_leaves_weights_untouched_until_first_gradient():
    wl = tiny_mlp(K=3, W=2)
    init = make_params(wl, 10)
    pipe = fdg.Pipeline(wl.ops, wl.bounds, wl.W, init, wl.lr)
    first_update = [2 * (3 - 1) - k0 for k0 in range(3)]  # iteration of the first non-zero gradient
    for t in range(7):
        pipe.step([make_batch(wl, 10, t, s) for s in range(wl.W)])
        for k0 in range(3):
            same = all(torch.equal(a, torch.as_tensor(b, dtype=DT)) for a, b in zip(pipe.w[0][k0], init[k0]))
            assert same == (t < first_update[k0]), (t, k0)
    assert pipe.loss is not None


def test_loss_is_reported_for_batch_t_minus_K_plus_1():
    wl = tiny_mlp(K=3, W=2)
    pipe, losses = _run(wl, seed=11, T=4)
    assert losses[0] is None and losses[1] is None and losses[2] is not None
    # at iteration 2 all weights are still initial: loss equals a plain forward of batch 0
    mods = [[torch.as_tensor(p, dtype=DT) for p in m] for m in make_params(wl, 11)]
    ref = np.mean([float(fdg.definition_gradient(wl.ops, wl.bounds, mods, *make_batch(wl, 11, 0, s))[1])
                   for s in range(2)])
    assert abs(float(losses[2]) - ref) < 1e-13


# ------------------------------------------------------------------ consensus
def _ring_edges(S):
    return [(i, (i + 1) % S) for i in range(S)] if S > 2 else [(0, 1)]


def test_gossip_matrix_properties():
    for S, edges, alpha in [(4, _ring_edges(4), 0.3), (5, [(0, 1), (1, 2), (2, 3), (3, 4)], 0.4),
                            (4, [(i, j) for i in range(4) for j in range(i + 1, 4)], 0.25)]:
        P = fdg.gossip_matrix(S, edges, alpha)
        assert torch.equal(P, P.t())
        assert torch.allclose(P.sum(0), torch.ones(S, dtype=DT)) and torch.allclose(P.sum(1), torch.ones(S, dtype=DT))
        gamma = torch.linalg.eigvalsh(P - torch.full((S, S), 1.0 / S, dtype=DT)).abs().max()
        assert float(gamma) < 1.0
    assert torch.allclose(fdg.gossip_matrix(4, [(i, j) for i in range(4) for j in range(i + 1, 4)], 0.25),
                          fdg.mean_matrix(4))


def test_disagreement_measure_on_hand_worked_cases():
    """delta of the experiment section, written out by hand on integer weights: the maximum over layers
    and data-groups of the Euclidean distance between a data-group's layer weight vector (weight AND bias,
    Section 2.1's w_l) and the average of that vector over the data-groups."""
    t = lambda v: torch.tensor(v, dtype=DT)
    # two data-groups, one module with two layers
    g0 = [[t([[1, 2], [3, 4]]), t([0, 2]), t([[5]]), t([1])]]
    g1 = [[t([[3, 2], [3, 0]]), t([2, 2]), t([[1]]), t([1])]]
    # layer A: mean weight [[2,2],[3,2]], mean bias [1,2]; deviations +-([[1,0],[0,2]], [1,0]): norm sqrt(1+4+1)
    # layer B: mean 3 / 1; deviations +-2 / 0: norm 2
    assert abs(fdg.consensus_error([g0, g1]) - 6 ** 0.5) < 1e-15
    # three data-groups, two modules; the largest deviation sits in module 1 and in the bias as much as the weight
    a = [[t([0, 0]), t([0])], [t([0, 0]), t([0])]]
    b = [[t([0, 0]), t([0])], [t([3, 0]), t([0])]]
    c = [[t([0, 0]), t([0])], [t([0, 3]), t([3])]]
    # module 1: mean weight [1,1], mean bias 1; deviations a: ([-1,-1],-1) -> sqrt 3; b: ([2,-1],-1) -> sqrt 6;
    # c: ([-1,2],2) -> 3. Per tensor the maximum would be sqrt 5, without the root 9, with a mean over groups ~2.4.
    assert abs(fdg.consensus_error([a, b, c]) - 3.0) < 1e-15
    assert fdg.consensus_error([a, a, a]) == 0.0


def test_exact_mean_keeps_replicas_identical():
    wl = tiny_resnet(K=2, W=3)
    pipe, _ = _run(wl, seed=12, T=7)
    assert fdg.consensus_error(pipe.w) < 1e-15
    assert any(not torch.equal(a, torch.as_tensor(b, dtype=DT))
               for a, b in zip(pipe.w[0][0], make_params(wl, 12)[0]))


def test_average_dynamics_and_consensus_bound_under_sparse_gossip():
    """Doubly stochastic P: the data-group average moves by -(lr/S) sum_s grad_s
    (Appendix A), and the disagreement contracts with gamma from a non-zero start."""
    wl = tiny_mlp(K=2, W=4)
    S = 4
    P = fdg.gossip_matrix(S, _ring_edges(S), 0.3)
    base = make_params(wl, 13)
    rng = np.random.default_rng(0)
    init = [[[p + 0.05 * rng.standard_normal(p.shape).astype(np.float32) for p in m] for m in base]
            for _ in range(S)]
    pipe = fdg.Pipeline(wl.ops, wl.bounds, S, init, wl.lr, 0.0, None, P)
    for t in range(6):
        avg_before = [[sum(pipe.w[s][k0][j] for s in range(S)) / S for j in range(len(pipe.w[0][k0]))]
                      for k0 in range(2)]
        pipe.step([make_batch(wl, 13, t, s) for s in range(S)])
        for k0 in range(2):
            for j in range(len(avg_before[k0])):
                gsum = sum((pipe.grad_log[(t, s, k0)][j] if (t, s, k0) in pipe.grad_log else 0.0) for s in range(S))
                expect = avg_before[k0][j] - wl.lr / S * gsum
                now = sum(pipe.w[s][k0][j] for s in range(S)) / S
                assert torch.allclose(now, expect, rtol=1e-12, atol=1e-14)
    # with zero step size the disagreement decays at least as fast as gamma^t
    pipe0 = fdg.Pipeline(wl.ops, wl.bounds, S, init, 0.0, 0.0, None, P)
    gamma = float(torch.linalg.eigvalsh(P - torch.full((S, S), 1.0 / S, dtype=DT)).abs().max())

    def stacked_delta(p):
        tot = 0.0
        for k0 in range(2):
            for j in range(len(p.w[0][k0])):
                avg = sum(p.w[s][k0][j] for s in range(S)) / S
                tot += sum(float(((p.w[s][k0][j] - avg) ** 2).sum()) for s in range(S))
        return tot ** 0.5

    d0 = stacked_delta(pipe0)
    for t in range(5):
        pipe0.step([make_batch(wl, 13, t, s) for s in range(S)])
        assert stacked_delta(pipe0) <= gamma ** (t + 1) * d0 * (1 + 1e-9)


# ------------------------------------------------------------------ step sizes
def _step_size_rows():
    rows = []
    for line in open(os.path.join(GOLD, "step_size_strategies.txt")):
        if line.strip() and not line.startswith("#"):
            rule, t, eta = line.split()
            rows.append((rule, int(t), float(eta)))
    return rows


def test_step_size_rules_match_the_printed_values():
    rows = _step_size_rows()
    assert len(rows) >= 14
    for rule, t, eta in rows:
        assert fdg.step_size(rule, t, 0.1) == pytest.approx(eta, rel=1e-12), (rule, t)
    # Strategy II never increases; the diminishing rule decreases strictly and is square-summable
    # but not summable (partial sums grow like log T)
    etas = [fdg.step_size("piecewise", t) for t in range(0, 50000, 500)]
    assert all(a >= b for a, b in zip(etas, etas[1:]))
    dim = [fdg.step_size("diminishing", t) for t in range(2000)]
    assert all(a > b for a, b in zip(dim, dim[1:]))
    assert sum(d * d for d in dim) < 0.1 ** 2 * (math.pi ** 2 / 6)
    assert sum(dim) > 0.1 * math.log(2000)
