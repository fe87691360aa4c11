"""The training recurrence: data parallelism over S data-groups combined with the
fully decoupled parallel backpropagation over K modules (Section 3.3, update
(a)/(b) of the proposed framework; Algorithm 1 in Appendix D).

Notation: agent (s, k0) with k0 = k-1 zero-based. d[k0] is the per-leg delay of
module k0; the paper's schedule is d[k0] = K-1-k0. Module k0 forwards the
mini-batch sampled at tau at iteration tau+k0 and back-propagates it at iteration
tau+k0+2*d[k0] (Section 3.2: forward of batch t-k+1, backward of batch t-2K+k+1
at iteration t), using the weights it held at the forward (w_l(t-2K+2k)).

Readings taken where the text leaves a choice:
  * the local loss Phi_s is the plain mean over the data-group's mini-batch and
    `lr` multiplies it directly (the paper's eta_t |D_s|/N equals lr for equal
    partitions with lr = eta_t / S);
  * the sum over the neighbour set in the mixing step includes the agent itself
    (the stacked form (P kron I) in Appendix A uses the full matrix P);
  * what travels up the line is the gradient with respect to the receiving
    module's output activation h_{q_k} (the only quantity that closes the chain
    rule of Section 2.2);
  * momentum (not in the paper) is v <- mu v + g, u = w - lr v per agent, with the
    whole update skipped while the gradient is defined as zero (tau < 0).
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence

import torch

from . import network as N

DT = torch.float64


# ----------------------------------------------------------------------------- schedule
def paper_delays(K: int) -> List[int]:
    return [K - 1 - k0 for k0 in range(K)]


def check_delays(K: int, d: Sequence[int]) -> None:
    """The last module may use its own loss gradient at once (d >= 0); module k0
    needs the error gradient module k0+1 produced at least one iteration earlier."""
    if len(d) != K or d[K - 1] < 0:
        raise ValueError("bad delays")
    for k0 in range(K - 1):
        if d[k0] < d[k0 + 1] + 1:
            raise ValueError("delays violate causality")


def schedule(t: int, K: int, d: Optional[Sequence[int]] = None) -> List[dict]:
    """Integers that drive iteration t for every module (closed forms of Section 3.2).
    f / b: mini-batch ids forwarded / back-propagated (negative = idle);
    ring_depth R = 2d+1 slots of saved activations and weight snapshots;
    fwd_slot = t mod R is written by the forward, bwd_slot = (t-2d) mod R is read
    by the backward; err_depth / err_write / err_read index the error-gradient
    mailbox between module k0+1 (writer) and k0 (reader); label_slot indexes the
    queue (depth K + 2 d[K-1]) of targets travelling to the last module.
    Further integers an implementation with shared storage needs, all consequences of
    the above: in_fwd_slot / in_bwd_slot = the slot of module k0-1's ring that holds the
    output module k0-1 produced for mini-batch f / b (it forwarded that batch one
    iteration before module k0 did, i.e. at f+k0-1 / b+k0-1), -1 for module 0;
    snap_write = (t+1) mod R, where the weights after this iteration's update are
    snapshotted (they are the ones the forward of iteration t+1 uses);
    label_write = t mod queue depth for module 0 (targets of the batch sampled now);
    label_bwd_slot = b mod queue depth for the last module (targets of the batch whose
    loss gradient starts this iteration's backward), -1 otherwise."""
    d = paper_delays(K) if d is None else list(d)
    out = []
    for k0 in range(K):
        R = 2 * d[k0] + 1
        f = t - k0
        b = t - k0 - 2 * d[k0]
        rec = {"k0": k0, "f": f, "b": b, "ring_depth": R, "fwd_slot": t % R,
               "bwd_slot": (t - 2 * d[k0]) % R}
        if k0 < K - 1:
            lag = 2 * (d[k0] - d[k0 + 1]) - 1  # iterations between producer and consumer
            rec["err_depth"] = lag + 1
            rec["err_read"] = (t - lag) % (lag + 1)   # slot the producer wrote `lag` steps ago
        else:
            rec["err_depth"] = 0
            rec["err_read"] = -1
        if k0 > 0:
            lag_up = 2 * (d[k0 - 1] - d[k0]) - 1
            rec["err_write"] = t % (lag_up + 1)
        else:
            rec["err_write"] = -1
        depth = K + 2 * d[K - 1]
        rec["label_slot"] = (f % depth) if (k0 == K - 1 and f >= 0) else -1
        if k0 > 0:
            R_up = 2 * d[k0 - 1] + 1
            rec["in_fwd_slot"] = ((f + k0 - 1) % R_up) if f >= 0 else -1
            rec["in_bwd_slot"] = ((b + k0 - 1) % R_up) if b >= 0 else -1
        else:
            rec["in_fwd_slot"] = rec["in_bwd_slot"] = -1
        rec["snap_write"] = (t + 1) % R
        rec["label_write"] = (t % depth) if k0 == 0 else -1
        rec["label_bwd_slot"] = (b % depth) if (k0 == K - 1 and b >= 0) else -1
        out.append(rec)
    return out


# ----------------------------------------------------------------------------- step sizes
def step_size(rule: str, t: int, eta0: float = 0.1) -> float:
    """eta_t of the experiment section (Strategy I "constant", Strategy II "piecewise") and of
    the diminishing step-size section ("diminishing": eta0 / (t + 1))."""
    if rule == "constant":
        return eta0
    if rule == "piecewise":
        if t <= 15000:
            return eta0
        if t <= 30000:
            return eta0 * 0.1
        if t <= 40000:
            return eta0 * 0.01
        return eta0 * 0.001
    if rule == "diminishing":
        return eta0 / (t + 1)
    raise ValueError(rule)


# ----------------------------------------------------------------------------- graphs
def gossip_matrix(S: int, edges: Sequence[tuple], alpha: float) -> torch.Tensor:
    """Weighted matrix of a communication graph: alpha on edges, 1 - degree*alpha on
    the diagonal (Section 2.3)."""
    P = torch.zeros((S, S), dtype=DT)
    deg = [0] * S
    for i, j in edges:
        P[i, j] = alpha
        P[j, i] = alpha
        deg[i] += 1
        deg[j] += 1
    for i in range(S):
        P[i, i] = 1.0 - deg[i] * alpha
    return P


def mean_matrix(S: int) -> torch.Tensor:
    """Complete graph with alpha = 1/S: every entry 1/S, so mixing is the exact mean."""
    return torch.full((S, S), 1.0 / S, dtype=DT)


def consensus_error(weights) -> float:
    """Disagreement measure delta(t) of the experiment section: the maximum over layers l and
    data-groups s of || w_{s,l} - (1/S) sum_r w_{r,l} ||_2, where w_{s,l} is data-group s's
    weight vector of layer l in the sense of Section 2.1 (w_l in R^{d_l}: ALL parameters of
    the layer, i.e. weight and bias -- gamma and beta for a normalisation -- as one vector).
    weights[s][k0][j]: the flat canonical list of module k0, in which every layer
    contributes two consecutive tensors (weight, bias)."""
    S = len(weights)
    worst = 0.0
    for k0 in range(len(weights[0])):
        n = len(weights[0][k0])
        assert n % 2 == 0
        for j in range(0, n, 2):
            sq = [0.0] * S
            for part in (j, j + 1):
                avg = sum(weights[s][k0][part] for s in range(S)) / S
                for s in range(S):
                    sq[s] += float(((weights[s][k0][part] - avg) ** 2).sum())
            worst = max(worst, max(sq) ** 0.5)
    return worst


# ----------------------------------------------------------------------------- O-pipe
class Pipeline:
    """Algorithm 1 executed agent by agent. All agents read what the previous
    iteration left in the mailboxes; nothing computed in iteration t is consumed
    before iteration t+1 except by the agent that computed it."""

    def __init__(self, ops, bounds, S, init_params, lr, momentum=0.0, delays=None, P=None, q=None):
        # q: optional storage rounding handed to every forward / backward pass (diagnostic mode of
        # oracle.network; None = exact fp64, the contract)
        self.q = q
        self.ops = ops
        self.bounds = list(bounds)
        self.K = len(bounds) - 1
        self.S = S
        self.d = paper_delays(self.K) if delays is None else list(delays)
        check_delays(self.K, self.d)
        self.lr = lr
        self.mu = momentum
        self.P = mean_matrix(S) if P is None else P.to(DT)
        # w[s][k0] = list of tensors; identical initial copies (delta(0) = 0) unless the
        # caller passes per-data-group initial weights as init_params[s][k0]
        if isinstance(init_params[0][0], (list, tuple)):
            self.w = [[[torch.as_tensor(p, dtype=DT).clone() for p in init_params[s][k0]]
                       for k0 in range(self.K)] for s in range(S)]
        else:
            self.w = [[[torch.as_tensor(p, dtype=DT).clone() for p in init_params[k0]]
                       for k0 in range(self.K)] for _ in range(S)]
        self.v = [[[torch.zeros_like(p) for p in self.w[s][k0]] for k0 in range(self.K)]
                  for s in range(S)]
        self.t = 0
        self.inflight = [[{} for _ in range(self.K)] for _ in range(S)]  # batch id -> (saved, weights)
        self.act_mail = [[None] * self.K for _ in range(S)]   # act_mail[s][k0]: input waiting for k0
        self.err_mail = [[{} for _ in range(self.K)] for _ in range(S)]  # err_mail[s][k0][batch] from k0+1
        self.labels = [{} for _ in range(S)]
        self.history = []   # history[t][s][k0] = weights at the start of iteration t
        self.grad_log = {}  # (t, s, k0) -> grads applied at iteration t
        self.loss = None
        self.keep_history = True

    def module_ops(self, k0):
        return self.ops[self.bounds[k0]:self.bounds[k0 + 1]]

    def step(self, batches):
        """batches[s] = (x [B,C,H,W], y [B]) sampled by agent (s,1) at this iteration."""
        t, K, S = self.t, self.K, self.S
        if self.keep_history:
            self.history.append([[list(self.w[s][k0]) for k0 in range(K)] for s in range(S)])
        new_act = [[None] * K for _ in range(S)]
        new_err = []  # (s, k0, batch, tensor) to post after every agent has run
        grads = [[None] * K for _ in range(S)]
        losses = []
        for s in range(S):
            x, y = batches[s]
            self.labels[s][t] = torch.as_tensor(y, dtype=torch.int64)
            for k0 in range(K):
                ops = self.module_ops(k0)
                last = k0 == K - 1
                f = t - k0
                b = t - k0 - 2 * self.d[k0]
                # forward of batch f with the current weights
                if f >= 0:
                    hin = torch.as_tensor(x, dtype=DT) if k0 == 0 else self.act_mail[s][k0]
                    out, saved, loss = N.forward(ops, self.w[s][k0], hin,
                                                 self.labels[s][f] if last else None, q=self.q)
                    self.inflight[s][k0][f] = (saved, self.w[s][k0], out if last else None)
                    if last:
                        losses.append(loss)
                        self.labels[s].pop(f)
                    else:
                        new_act[s][k0 + 1] = out
                # backward of batch b with the weights of its forward
                if b >= 0:
                    saved, w_old, dlogits = self.inflight[s][k0].pop(b)
                    dout = dlogits if last else self.err_mail[s][k0].pop(b)
                    dx, g = N.backward(ops, w_old, saved, dout, need_dx=(k0 > 0), q=self.q)
                    grads[s][k0] = g
                    if k0 > 0:
                        new_err.append((s, k0 - 1, b, dx))
        # hand-offs become visible at the next iteration
        for s in range(S):
            for k0 in range(1, K):
                self.act_mail[s][k0] = new_act[s][k0]
        for s, k0, b, dx in new_err:
            self.err_mail[s][k0][b] = dx
        # u_{s,k} = w_{s,k} - lr * grad (zero gradient: u = w), then w_{s,k} <- sum_r P_sr u_{r,k}
        for k0 in range(K):
            u = []
            for s in range(S):
                g = grads[s][k0]
                if g is None:
                    u.append(self.w[s][k0])
                    continue
                self.grad_log[(t, s, k0)] = g
                if self.mu != 0.0:
                    self.v[s][k0] = [self.mu * v + gi for v, gi in zip(self.v[s][k0], g)]
                    direction = self.v[s][k0]
                else:
                    direction = g
                u.append([w - self.lr * di for w, di in zip(self.w[s][k0], direction)])
            for s in range(S):
                self.w[s][k0] = [sum(self.P[s, r] * u[r][j] for r in range(S))
                                 for j in range(len(u[s]))]
        self.loss = (sum(losses) / len(losses)) if losses else None
        self.t += 1
        return self.loss

    def params(self, s=0):
        return [[p.clone() for p in self.w[s][k0]] for k0 in range(self.K)]


# ----------------------------------------------------------------------------- O-def
def definition_gradient(ops, bounds, skewed_weights, x, y, q=None):
    """Ordinary (locked) backpropagation of the whole network on one mini-batch at
    the weight vector `skewed_weights` (list over modules of param lists).
    Returns grads[k0] aligned with skewed_weights[k0] and the loss.
    q: optional storage rounding (diagnostic mode of oracle.network)."""
    K = len(bounds) - 1
    h = torch.as_tensor(x, dtype=DT)
    saved_all = []
    loss = None
    for k0 in range(K):
        mops = ops[bounds[k0]:bounds[k0 + 1]]
        h, saved, l = N.forward(mops, skewed_weights[k0], h,
                                torch.as_tensor(y, dtype=torch.int64) if k0 == K - 1 else None, q=q)
        saved_all.append(saved)
        if l is not None:
            loss = l
    d = h
    grads = [None] * K
    for k0 in range(K - 1, -1, -1):
        mops = ops[bounds[k0]:bounds[k0 + 1]]
        d, grads[k0] = N.backward(mops, skewed_weights[k0], saved_all[k0], d, need_dx=(k0 > 0), q=q)
    return grads, loss


def definition_replay(ops, bounds, S, init_params, lr, momentum, delays, P,
                      batch_fn: Callable[[int, int], tuple], T: int):
    """The same recurrence evaluated from its definition: at iteration t agent (s,k0)
    applies the true gradient of the loss of mini-batch b = t-k0-2d[k0] at the skewed
    weight vector col{ w_{s,j}(b+j0) : j } (Section 3.3), obtained by an ordinary
    whole-network backward pass. Returns the weight history w[t][s][k0]."""
    K = len(bounds) - 1
    d = paper_delays(K) if delays is None else list(delays)
    P = mean_matrix(S) if P is None else P.to(DT)
    w = [[[torch.as_tensor(p, dtype=DT).clone() for p in init_params[k0]] for k0 in range(K)]
         for _ in range(S)]
    v = [[[torch.zeros_like(p) for p in w[s][k0]] for k0 in range(K)] for s in range(S)]
    hist = []
    for t in range(T):
        hist.append([[list(w[s][k0]) for k0 in range(K)] for s in range(S)])
        for k0 in range(K):
            b = t - k0 - 2 * d[k0]
            u = []
            for s in range(S):
                if b < 0:
                    u.append(w[s][k0])
                    continue
                skew = [hist[b + j0][s][j0] for j0 in range(K)]
                x, y = batch_fn(b, s)
                g_all, _ = definition_gradient(ops, bounds, skew, x, y)
                g = g_all[k0]
                if momentum != 0.0:
                    v[s][k0] = [momentum * vi + gi for vi, gi in zip(v[s][k0], g)]
                    direction = v[s][k0]
                else:
                    direction = g
                u.append([wi - lr * di for wi, di in zip(w[s][k0], direction)])
            new = [[sum(P[s, r] * u[r][j] for r in range(S)) for j in range(len(u[s]))]
                   for s in range(S)]
            for s in range(S):
                w[s][k0] = new[s]
    hist.append([[list(w[s][k0]) for k0 in range(K)] for s in range(S)])
    return hist
