"""Network descriptions for the five benchmark configurations (pure data).

An op record is a dict with key "op" in
  conv      : cin, cout, k, stride, pad      (2-D convolution + bias)
  linear    : cin, cout                      (dense layer + bias, on [N, cin, 1, 1])
  bn        : c, eps                         (training-mode batch normalisation per data-group:
                                              statistics over that group's mini-batch; gamma, beta)
  relu
  maxpool2                                   (2x2 window, stride 2)
  gap                                        (global average pool -> [N, C, 1, 1])
  res_begin                                  (remember the current tensor as block input)
  res_add   : scale, shortcut                (y = shortcut(x_in) + scale * y_main;
                                              shortcut is None (identity) or a dict
                                              cin, cout, k, stride, pad of a conv + bias)
  softmax_ce                                 (mean softmax cross-entropy, last op)

`bounds` has K+1 indices into the op list: module k0 owns ops[bounds[k0]:bounds[k0+1]].
The residual networks are BatchNorm-free: every block output is
relu(shortcut(x) + scale * (conv2(relu(conv1(x))))), scale = 1/sqrt(number of blocks).
"""
from __future__ import annotations

import copy
import math
from dataclasses import dataclass, field
from typing import List, Optional


@dataclass
class Workload:
    name: str
    ops: List[dict]
    bounds: List[int]
    K: int
    W: int
    B: int
    in_shape: tuple  # (C, H, W) of one sample as the caller lays it out (NCHW)
    classes: int
    precision: str  # "f32" | "bf16"  (bf16 = bf16 activations/weights + fp32 master)
    lr: float
    momentum: float
    steps: int
    delays: Optional[List[int]] = None  # None -> the paper's schedule d_k = K-1-k0
    notes: str = ""
    extra: dict = field(default_factory=dict)


def _conv(cin, cout, k=3, stride=1, pad=None):
    if pad is None:
        pad = (k - 1) // 2
    return {"op": "conv", "cin": cin, "cout": cout, "k": k, "stride": stride, "pad": pad}


def _linear(cin, cout):
    return {"op": "linear", "cin": cin, "cout": cout}


def _relu():
    return {"op": "relu"}


def _bn(c, eps=1e-5):
    return {"op": "bn", "c": c, "eps": eps}


def _block(cin, cout, stride, scale, bn=False):
    """relu(shortcut(x) + scale * conv2(relu(conv1(x)))); with bn: a batch normalisation after
    each of the two convolutions (the projection shortcut stays a plain convolution)."""
    sc = None
    if stride != 1 or cin != cout:
        sc = {"cin": cin, "cout": cout, "k": 1, "stride": stride, "pad": 0}
    norm = [_bn(cout)] if bn else []
    return [
        {"op": "res_begin"},
        _conv(cin, cout, 3, stride), *norm,
        _relu(),
        _conv(cout, cout, 3, 1), *norm,
        {"op": "res_add", "scale": scale, "shortcut": sc},
        _relu(),
    ]


def _mlp():
    ops = [
        _linear(3072, 256), _relu(),
        _linear(256, 256), _relu(),
        _linear(256, 10), {"op": "softmax_ce"},
    ]
    return Workload(
        name="cfg0_mlp", ops=ops, bounds=[0, 2, 4, 6], K=3, W=2, B=32,
        in_shape=(3072, 1, 1), classes=10, precision="f32", lr=0.01, momentum=0.0, steps=20,
        notes="32x32x3 image flattened in NCHW order to 3072 features",
    )


def _cnn():
    ops, bounds = [], [0]
    cin = 3
    for j, cout in enumerate((64, 128, 256, 512)):
        ops += [_conv(cin, cout), _relu(), {"op": "maxpool2"}]
        cin = cout
        if j < 3:
            bounds.append(len(ops))
    ops += [{"op": "gap"}, _linear(512, 10), {"op": "softmax_ce"}]
    bounds.append(len(ops))
    return Workload(
        name="cfg1_cnn", ops=ops, bounds=bounds, K=4, W=4, B=128, in_shape=(3, 32, 32),
        classes=10, precision="f32", lr=0.001, momentum=0.9, steps=100,
        notes="step size not given by the configuration; 0.01 with momentum 0.9 diverges on this "
              "BatchNorm-free net (loss 5 -> 500 in 12 updates), 0.001 does not",
    )


def _resnet(name, stem, stages, module_blocks, K, W, B, steps, lr=0.01, bn=False):
    """stages: list of (channels, n_blocks); module_blocks: blocks per module (len K).
    bn: the standard form (batch normalisation after every main-path convolution, residual
    branch added unscaled) instead of the normalisation-free one."""
    nblocks = sum(n for _, n in stages)
    assert sum(module_blocks) == nblocks and len(module_blocks) == K
    scale = 1.0 if bn else 1.0 / math.sqrt(nblocks)
    blocks = []
    cin = stem
    for si, (c, n) in enumerate(stages):
        for bi in range(n):
            stride = 2 if (bi == 0 and si > 0) else 1
            blocks.append(_block(cin, c, stride, scale, bn))
            cin = c
    ops = [_conv(3, stem), *([_bn(stem)] if bn else []), _relu()]
    bounds = [0]
    it = iter(blocks)
    for k0, nb in enumerate(module_blocks):
        for _ in range(nb):
            ops += next(it)
        if k0 < K - 1:
            bounds.append(len(ops))
    ops += [{"op": "gap"}, _linear(cin, 10), {"op": "softmax_ce"}]
    bounds.append(len(ops))
    return Workload(
        name=name, ops=ops, bounds=bounds, K=K, W=W, B=B, in_shape=(3, 32, 32), classes=10,
        precision="bf16", lr=lr, momentum=0.0, steps=steps,
        extra={"blocks": nblocks, "res_scale": scale},
    )


def _resnet18(bn=False):
    return _resnet("cfg2_resnet18" + ("_bn" if bn else ""), 64, [(64, 2), (128, 2), (256, 2), (512, 2)],
                   [2, 2, 2, 2], K=4, W=4, B=128, steps=16, bn=bn)


def _resnet56():
    cuts = [int(round(i * 27 / 8)) for i in range(9)]
    per_module = [cuts[i + 1] - cuts[i] for i in range(8)]
    return _resnet("cfg3_resnet56", 16, [(16, 9), (32, 9), (64, 9)], per_module,
                   K=8, W=8, B=128, steps=24)


def _resnet34w():
    return _resnet("cfg4_resnet34w", 128, [(128, 3), (256, 4), (512, 6), (1024, 3)],
                   [2] * 8, K=8, W=8, B=256, steps=24)


def _paper_resnet20(S, K, bn=False):
    """The network and batch of the paper's experiments (Section 5: ResNet-20, mini-batch 194 per
    data-group, S in {1, 4} data-groups, K in {1, 2} modules), BatchNorm-free like cfg2-4, on
    synthetic CIFAR-shaped data. K = 2 cuts after the fifth of the nine blocks."""
    return _resnet(f"paper_r20_S{S}K{K}" + ("_bn" if bn else ""), 16, [(16, 3), (32, 3), (64, 3)],
                   [9] if K == 1 else [5, 4], K=K, W=S, B=194, steps=2 * (K - 1) + 10, bn=bn)


_BUILDERS = {
    "cfg0_mlp": _mlp,
    "cfg1_cnn": _cnn,
    "cfg2_resnet18": _resnet18,
    "cfg3_resnet56": _resnet56,
    "cfg4_resnet34w": _resnet34w,
    "paper_r20_S1K1": lambda: _paper_resnet20(1, 1),
    "paper_r20_S1K2": lambda: _paper_resnet20(1, 2),
    "paper_r20_S4K1": lambda: _paper_resnet20(4, 1),
    "paper_r20_S4K2": lambda: _paper_resnet20(4, 2),
    # the same networks in their standard form, with training-mode batch normalisation
    "cfg2_resnet18_bn": lambda: _resnet18(bn=True),
    "paper_r20_S1K1_bn": lambda: _paper_resnet20(1, 1, bn=True),
    "paper_r20_S1K2_bn": lambda: _paper_resnet20(1, 2, bn=True),
    "paper_r20_S4K1_bn": lambda: _paper_resnet20(4, 1, bn=True),
    "paper_r20_S4K2_bn": lambda: _paper_resnet20(4, 2, bn=True),
}
WORKLOAD_NAMES = tuple(n for n in _BUILDERS if n.startswith("cfg") and not n.endswith("_bn"))  # the five benchmark configurations
PAPER_WORKLOAD_NAMES = tuple(n for n in _BUILDERS if n.startswith("paper_") and not n.endswith("_bn"))
BN_WORKLOAD_NAMES = tuple(n for n in _BUILDERS if n.endswith("_bn"))


def workload(name: str, *, B: Optional[int] = None, W: Optional[int] = None,
             steps: Optional[int] = None, precision: Optional[str] = None,
             lr: Optional[float] = None, momentum: Optional[float] = None) -> Workload:
    """Return a fresh copy of a named configuration, optionally with a reduced
    per-replica batch / replica count / step count (used by parity tests whose
    oracle leg must finish in seconds)."""
    wl = copy.deepcopy(_BUILDERS[name]())
    if B is not None:
        wl.B = B
    if W is not None:
        wl.W = W
    if steps is not None:
        wl.steps = steps
    if precision is not None:
        wl.precision = precision
    if lr is not None:
        wl.lr = lr
    if momentum is not None:
        wl.momentum = momentum
    return wl


def tiny_resnet(K=2, W=2, B=4, hw=8, c=8, precision="f32", steps=8, bn=False) -> Workload:
    """A 3-block residual net on hw x hw images (one projection block), small
    enough for finite differences and exhaustive checks."""
    scale = 1.0 / math.sqrt(3)
    ops = [_conv(3, c), *([_bn(c)] if bn else []), _relu()]
    ops += _block(c, c, 1, scale, bn)
    cut = len(ops)
    ops += _block(c, 2 * c, 2, scale, bn)
    nb2 = len(ops) - cut
    ops += _block(2 * c, 2 * c, 1, scale, bn)
    ops += [{"op": "gap"}, _linear(2 * c, 10), {"op": "softmax_ce"}]
    if K == 1:
        bounds = [0, len(ops)]
    elif K == 2:
        bounds = [0, cut, len(ops)]
    elif K == 3:
        bounds = [0, cut, cut + nb2, len(ops)]
    else:
        raise ValueError("tiny_resnet supports K in 1..3")
    return Workload(name=f"tiny_resnet_K{K}" + ("_bn" if bn else ""), ops=ops, bounds=bounds, K=K, W=W, B=B,
                    in_shape=(3, hw, hw), classes=10, precision=precision, lr=0.05,
                    momentum=0.0, steps=steps, extra={"blocks": 3, "res_scale": scale})


def odd_resnet(precision="f32", K=2, W=2, B=3, h=7, w=9, c=16, steps=8) -> Workload:
    """Awkward shapes on purpose: odd image sides (so a stride-2 block halves 7 x 9 to 4 x 5), an odd
    per-replica batch, a projection block whose channel counts still reach the stride-2 dgrad path
    that folds the shortcut in, and a 10-channel 1x1 conv whose channel stride is padded."""
    scale = 1.0 / math.sqrt(2)
    ops = [_conv(3, c), _relu()]
    ops += _block(c, 2 * c, 2, scale)
    cut = len(ops)
    ops += _block(2 * c, 2 * c, 1, scale)
    ops += [_conv(2 * c, 10, 1, 1), _relu(), {"op": "gap"}, _linear(10, 10), {"op": "softmax_ce"}]
    bounds = [0, len(ops)] if K == 1 else [0, cut, len(ops)]
    return Workload(name=f"odd_resnet_K{K}", ops=ops, bounds=bounds, K=K, W=W, B=B,
                    in_shape=(3, h, w), classes=10, precision=precision, lr=0.05,
                    momentum=0.0, steps=steps, extra={"blocks": 2, "res_scale": scale})


def tiny_cnn(K=2, W=2, B=4, hw=8, c=4, precision="f32", steps=8, momentum=0.9, bn=False) -> Workload:
    """conv-relu-maxpool x2, gap, linear: the cfg1 structure at toy size (bn: a batch normalisation
    after each convolution)."""
    ops = [_conv(3, c), *([_bn(c)] if bn else []), _relu(), {"op": "maxpool2"}]
    cut = len(ops)
    ops += [_conv(c, 2 * c), *([_bn(2 * c)] if bn else []), _relu(), {"op": "maxpool2"}, {"op": "gap"},
            _linear(2 * c, 10), {"op": "softmax_ce"}]
    bounds = [0, len(ops)] if K == 1 else [0, cut, len(ops)]
    return Workload(name=f"tiny_cnn_K{K}" + ("_bn" if bn else ""), ops=ops, bounds=bounds, K=K, W=W, B=B,
                    in_shape=(3, hw, hw), classes=10, precision=precision, lr=0.05,
                    momentum=momentum, steps=steps)


def uneven_cnn(W=2, B=128, hw=16, precision="bf16", steps=2) -> Workload:
    """3 -> 32 -> 128 -> 64 channels, stride 1, one module: layers whose input and output widths differ by
    a factor of two to four, at a pixel count (W * B * hw * hw >= 65536) that selects the large pixel tiles."""
    ops = [_conv(3, 32), _relu(), _conv(32, 128), _relu(), _conv(128, 64), _relu(), {"op": "gap"},
           _linear(64, 10), {"op": "softmax_ce"}]
    return Workload(name="uneven_cnn", ops=ops, bounds=[0, len(ops)], K=1, W=W, B=B, in_shape=(3, hw, hw),
                    classes=10, precision=precision, lr=0.05, momentum=0.0, steps=steps)


def tiny_mlp(K=3, W=2, B=4, feat=12, hidden=8, precision="f32", steps=10) -> Workload:
    """K linear layers (ReLU between), one per module: the cfg0 structure at toy size."""
    ops, bounds = [], [0]
    cin = feat
    for k0 in range(K):
        last = k0 == K - 1
        ops.append(_linear(cin, 10 if last else hidden))
        ops.append({"op": "softmax_ce"} if last else _relu())
        cin = hidden
        bounds.append(len(ops))
    return Workload(name=f"tiny_mlp_K{K}", ops=ops, bounds=bounds, K=K, W=W, B=B,
                    in_shape=(feat, 1, 1), classes=10, precision=precision, lr=0.05,
                    momentum=0.0, steps=steps)


# ----------------------------------------------------------------------------- communication graphs
def ring_mixing(W: int, alpha: float):
    """Mixing matrix of a ring of W data-groups (Section 2.3): alpha towards each of the two
    neighbours, the rest on the diagonal. W = 2 is a single edge. Returned as nested lists."""
    P = [[0.0] * W for _ in range(W)]
    edges = {(i, (i + 1) % W) for i in range(W)} if W > 2 else ({(0, 1)} if W == 2 else set())
    for i, j in edges:
        P[i][j] += alpha
        P[j][i] += alpha
    for i in range(W):
        P[i][i] = 1.0 - sum(P[i][j] for j in range(W) if j != i)
    return P


def complete_mixing(W: int):
    """Complete graph with weight 1/W everywhere: the exact mean."""
    return [[1.0 / W] * W for _ in range(W)]
