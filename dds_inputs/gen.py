"""Counter-seeded synthetic inputs: mini-batches and initial weights.

Stand-ins for CIFAR-10 shaped data: pixels i.i.d. N(0,1) float32 in NCHW order,
labels uniform integers in [0, classes). Every (seed, t, s) names its own stream,
so any batch can be regenerated in isolation.
"""
from __future__ import annotations

import math
from typing import List, Tuple

import numpy as np

_PARAM_STREAM = 10 ** 6


def make_batch(wl, seed: int, t: int, s: int) -> Tuple[np.ndarray, np.ndarray]:
    """Mini-batch sampled by replica s at iteration t: (x [B,C,H,W] f32, y [B] i32)."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, t, s])))
    c, h, w = wl.in_shape
    x = rng.standard_normal((wl.B, c, h, w), dtype=np.float32)
    y = rng.integers(0, wl.classes, size=(wl.B,), dtype=np.int32)
    return x, y


def param_shapes(ops) -> List[Tuple[str, tuple, int]]:
    """Canonical parameter tensors of an op list, in order: (name, shape, fan_in).
    conv: weight [cout,cin,k,k] then bias [cout]; linear: weight [cout,cin] then bias;
    bn: gamma [c] (fan_in -1) then beta [c] (fan_in -2);
    res_add with a projection shortcut: its conv weight then bias."""
    out = []
    for i, op in enumerate(ops):
        kind = op["op"]
        if kind == "conv":
            k = op["k"]
            out.append((f"{i}.conv.weight", (op["cout"], op["cin"], k, k), op["cin"] * k * k))
            out.append((f"{i}.conv.bias", (op["cout"],), 0))
        elif kind == "linear":
            out.append((f"{i}.linear.weight", (op["cout"], op["cin"]), op["cin"]))
            out.append((f"{i}.linear.bias", (op["cout"],), 0))
        elif kind == "bn":
            out.append((f"{i}.bn.weight", (op["c"],), -1))
            out.append((f"{i}.bn.bias", (op["c"],), -2))
        elif kind == "res_add" and op.get("shortcut"):
            sc = op["shortcut"]
            k = sc["k"]
            out.append((f"{i}.shortcut.weight", (sc["cout"], sc["cin"], k, k), sc["cin"] * k * k))
            out.append((f"{i}.shortcut.bias", (sc["cout"],), 0))
    return out


def make_params(wl, seed: int) -> List[List[np.ndarray]]:
    """Initial weights per module (list over modules of lists of float32 arrays in
    canonical order). Weights ~ N(0, 2/fan_in), biases zero; batch-norm gamma ~ 1 + 0.1 N(0,1),
    beta ~ 0.1 N(0,1) (away from the usual 1 / 0 so that a swapped or dropped one shows)."""
    mods = []
    for k0 in range(wl.K):
        ops = wl.ops[wl.bounds[k0]:wl.bounds[k0 + 1]]
        tensors = []
        for j, (_, shape, fan_in) in enumerate(param_shapes(ops)):
            if fan_in == 0:
                tensors.append(np.zeros(shape, dtype=np.float32))
            else:
                rng = np.random.Generator(
                    np.random.PCG64(np.random.SeedSequence([seed, _PARAM_STREAM, k0, j])))
                if fan_in < 0:
                    base = np.float32(1.0 if fan_in == -1 else 0.0)
                    tensors.append(base + rng.standard_normal(shape, dtype=np.float32) * np.float32(0.1))
                    continue
                std = math.sqrt(2.0 / fan_in)
                tensors.append((rng.standard_normal(shape, dtype=np.float32) * np.float32(std)))
        mods.append(tensors)
    return mods
