"""ctypes binding of libdds.so: argument marshalling only.

Every function of include/dds.h is exposed under the same name. `Trainer` bundles a
context with the arena tensor that backs it; PyTorch is used for device memory and
the current stream, nothing else. There is no CPU fallback: importing this module
without the built library, or constructing a Trainer without a GPU, raises.
"""
from __future__ import annotations

import ctypes as C
import math
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdds.so")

DDS_OK, DDS_EINVAL, DDS_ENOMEM, DDS_EHIP, DDS_EUNSUPPORTED = 0, -1, -2, -3, -4
DDS_SCHED_INTS = 13
OPS = {"conv": 1, "linear": 2, "relu": 3, "maxpool2": 4, "gap": 5, "res_begin": 6, "res_add": 7,
       "softmax_ce": 8, "bn": 9}
PRECISION = {"f32": 0, "bf16": 1}
ACTIVATIONS = {"store": 0, "recompute": 1}  # dds_spec.activations

EXPORTS = ["dds_schedule", "dds_step_size", "dds_arena_bytes", "dds_create", "dds_destroy", "dds_param_count",
           "dds_get_params", "dds_set_params", "dds_get_params_replica", "dds_consensus_error", "dds_consensus_error_static", "dds_step", "dds_get_loss", "dds_step_count",
           "dds_launches_last_step", "dds_gemm_flops_per_step", "dds_profile", "dds_profile_read",
           "dds_debug_bytes", "dds_debug_read", "dds_last_error"]


class dds_layer(C.Structure):
    _fields_ = [("op", C.c_int32), ("cin", C.c_int32), ("cout", C.c_int32), ("ksize", C.c_int32),
                ("stride", C.c_int32), ("pad", C.c_int32), ("res_scale", C.c_float),
                ("reserved", C.c_int32)]


class dds_spec(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("layers", C.POINTER(dds_layer)),
                ("bounds", C.POINTER(C.c_int32)), ("in_c", C.c_int32), ("in_h", C.c_int32),
                ("in_w", C.c_int32), ("classes", C.c_int32), ("batch", C.c_int32),
                ("precision", C.c_int32), ("lr", C.c_float), ("momentum", C.c_float),
                ("mixing", C.POINTER(C.c_float)), ("activations", C.c_int32)]


class DdsError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"dds error {code}: {msg}")
        self.code = code


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
    # The arena and the streams handed to the library come from PyTorch, so both must talk to
    # one HIP runtime: load PyTorch's first, libdds.so then binds to it by soname. (Loaded the
    # other way round the process holds two runtimes and the second finds no device.)
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i32p, f32p = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_float)
    lib.dds_schedule.argtypes = [C.c_int, C.POINTER(C.c_int), C.c_int64, i32p]
    lib.dds_step_size.argtypes = [C.c_int, C.c_int64, C.c_float]
    lib.dds_step_size.restype = C.c_float
    lib.dds_arena_bytes.argtypes = [C.POINTER(dds_spec), C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_size_t)]
    lib.dds_create.argtypes = [C.POINTER(dds_spec), C.c_int, C.c_int, C.POINTER(C.c_int), vp, C.c_size_t, C.POINTER(vp)]
    lib.dds_destroy.argtypes = [vp]
    lib.dds_param_count.argtypes = [vp, C.c_int]
    lib.dds_param_count.restype = C.c_int64
    lib.dds_get_params.argtypes = [vp, C.c_int, vp, C.c_size_t, vp]
    lib.dds_set_params.argtypes = [vp, C.c_int, vp, C.c_size_t, vp]
    lib.dds_get_params_replica.argtypes = [vp, C.c_int, C.c_int, vp, C.c_size_t, vp]
    lib.dds_consensus_error.argtypes = [vp, C.POINTER(C.c_double), vp]
    lib.dds_consensus_error_static.argtypes = [vp, C.POINTER(C.c_double), vp]
    lib.dds_step.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), C.c_float, vp]
    lib.dds_get_loss.argtypes = [vp, f32p, vp]
    lib.dds_step_count.argtypes = [vp]
    lib.dds_step_count.restype = C.c_int64
    lib.dds_launches_last_step.argtypes = [vp]
    lib.dds_launches_last_step.restype = C.c_int64
    lib.dds_gemm_flops_per_step.argtypes = [vp]
    lib.dds_gemm_flops_per_step.restype = C.c_double
    lib.dds_profile.argtypes = [vp, C.c_int]
    lib.dds_profile_read.argtypes = [vp, C.POINTER(C.c_double)]
    lib.dds_debug_bytes.argtypes = [vp, C.c_int, C.c_int, C.c_int]
    lib.dds_debug_bytes.restype = C.c_int64
    lib.dds_debug_read.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.c_int, vp, C.c_size_t, vp]
    lib.dds_last_error.restype = C.c_char_p
    return lib


lib = _load()


def _check(rc):
    if rc != DDS_OK:
        raise DdsError(rc, lib.dds_last_error().decode())


def _delays_arg(delays, K):
    if delays is None:
        return None
    assert len(delays) == K
    return (C.c_int * K)(*delays)


DDS_ETA_CONSTANT, DDS_ETA_PIECEWISE, DDS_ETA_DIMINISHING = 1, 2, 3
DDS_DBG_INPUT, DDS_DBG_OUTPUT, DDS_DBG_ERROR, DDS_DBG_LABELS, DDS_DBG_SNAPSHOT = 0, 1, 2, 3, 4


def dds_step_size(rule: int, t: int, eta0: float) -> float:
    return float(lib.dds_step_size(rule, t, eta0))


def dds_schedule(K: int, delays: Optional[Sequence[int]], t: int) -> np.ndarray:
    out = np.zeros((K, DDS_SCHED_INTS), dtype=np.int32)
    _check(lib.dds_schedule(K, _delays_arg(delays, K), t, out.ctypes.data_as(C.POINTER(C.c_int32))))
    return out


class Spec:
    """Owns the ctypes arrays behind a dds_spec."""

    def __init__(self, ops, bounds, in_shape, classes, batch, precision, lr, momentum, mixing=None, activations="store"):
        n = len(ops)
        self.layers = (dds_layer * n)()
        for i, op in enumerate(ops):
            L = self.layers[i]
            L.op = OPS[op["op"]]
            if op["op"] == "conv":
                L.cin, L.cout, L.ksize, L.stride, L.pad = op["cin"], op["cout"], op["k"], op["stride"], op["pad"]
            elif op["op"] == "linear":
                L.cin, L.cout, L.ksize, L.stride, L.pad = op["cin"], op["cout"], 1, 1, 0
            elif op["op"] == "bn":
                L.cin = L.cout = op["c"]
                L.res_scale = op["eps"]
            elif op["op"] == "res_add":
                L.res_scale = op["scale"]
                sc = op.get("shortcut")
                if sc:
                    L.cin, L.cout, L.ksize, L.stride, L.pad = sc["cin"], sc["cout"], sc["k"], sc["stride"], sc["pad"]
        self.bounds = (C.c_int32 * len(bounds))(*bounds)
        self.K = len(bounds) - 1
        # mixing: None (exact mean) or a W x W array, the matrix P of the communication graph
        self.mixing = None
        if mixing is not None:
            flat = np.ascontiguousarray(np.asarray(mixing, dtype=np.float32)).ravel()
            self.mixing = (C.c_float * flat.size)(*flat.tolist())
        self.c = dds_spec(n, self.layers, self.bounds, in_shape[0], in_shape[1], in_shape[2], classes, batch,
                          PRECISION[precision], lr, momentum, self.mixing, ACTIVATIONS[activations])

    @classmethod
    def from_workload(cls, wl, mixing=None, activations="store"):
        return cls(wl.ops, wl.bounds, wl.in_shape, wl.classes, wl.B, wl.precision, wl.lr, wl.momentum, mixing, activations)


def dds_arena_bytes(spec: Spec, K: int, W: int, delays=None) -> int:
    n = C.c_size_t(0)
    _check(lib.dds_arena_bytes(C.byref(spec.c), K, W, _delays_arg(delays, K), C.byref(n)))
    return n.value


class Trainer:
    """A dds context plus the device arena that backs it."""

    def __init__(self, spec: Spec, W: int, delays=None, device="cuda:0"):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("dds needs a GPU: there is no CPU path")
        self.torch = torch
        self.spec, self.K, self.W = spec, spec.K, W
        self.device = torch.device(device)
        nbytes = dds_arena_bytes(spec, self.K, W, delays)
        self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = (self.arena.data_ptr() + 255) // 256 * 256
        ctx = C.c_void_p()
        _check(lib.dds_create(C.byref(spec.c), self.K, W, _delays_arg(delays, self.K), base, nbytes, C.byref(ctx)))
        self.ctx = ctx
        self.arena_bytes = nbytes

    def _stream(self):
        return C.c_void_p(self.torch.cuda.current_stream(self.device).cuda_stream)

    def dds_param_count(self, module: int) -> int:
        n = lib.dds_param_count(self.ctx, module)
        if n < 0:
            _check(int(n))
        return int(n)

    def dds_set_params(self, module: int, tensors: Sequence[np.ndarray]):
        flat = np.concatenate([np.asarray(t, dtype=np.float32).ravel() for t in tensors])
        dev = self.torch.from_numpy(flat).to(self.device)
        _check(lib.dds_set_params(self.ctx, module, dev.data_ptr(), flat.size, self._stream()))
        self.torch.cuda.synchronize(self.device)

    def dds_get_params(self, module: int) -> np.ndarray:
        n = self.dds_param_count(module)
        dev = self.torch.empty(n, dtype=self.torch.float32, device=self.device)
        _check(lib.dds_get_params(self.ctx, module, dev.data_ptr(), n, self._stream()))
        self.torch.cuda.synchronize(self.device)
        return dev.cpu().numpy()

    def dds_get_params_replica(self, module: int, replica: int) -> np.ndarray:
        n = self.dds_param_count(module)
        dev = self.torch.empty(n, dtype=self.torch.float32, device=self.device)
        _check(lib.dds_get_params_replica(self.ctx, module, replica, dev.data_ptr(), n, self._stream()))
        self.torch.cuda.synchronize(self.device)
        return dev.cpu().numpy()

    def dds_consensus_error(self) -> float:
        v = C.c_double()
        _check(lib.dds_consensus_error(self.ctx, C.byref(v), self._stream()))
        return v.value

    def dds_consensus_error_static(self) -> float:
        v = C.c_double()
        _check(lib.dds_consensus_error_static(self.ctx, C.byref(v), self._stream()))
        return v.value

    def dds_step(self, xs, ys, lr: float = math.nan):
        """xs[s]: float32 CUDA tensor [B,C,H,W]; ys[s]: int32 CUDA tensor [B]."""
        W = self.W
        xp = (C.c_void_p * W)(*[x.data_ptr() for x in xs])
        yp = (C.c_void_p * W)(*[y.data_ptr() for y in ys])
        _check(lib.dds_step(self.ctx, xp, yp, lr, self._stream()))

    def dds_get_loss(self) -> float:
        v = C.c_float()
        _check(lib.dds_get_loss(self.ctx, C.byref(v), self._stream()))
        return v.value

    def dds_step_count(self) -> int:
        return int(lib.dds_step_count(self.ctx))

    def dds_launches_last_step(self) -> int:
        return int(lib.dds_launches_last_step(self.ctx))

    def dds_gemm_flops_per_step(self) -> float:
        return float(lib.dds_gemm_flops_per_step(self.ctx))

    def dds_debug_read(self, what: int, module: int, slot: int, index: int = 0) -> np.ndarray:
        """Raw bytes of one delay-buffer region (see include/dds.h) as a uint8 array."""
        n = lib.dds_debug_bytes(self.ctx, what, module, index)
        if n < 0:
            _check(int(n))
        dev = self.torch.empty(int(n), dtype=self.torch.uint8, device=self.device)
        _check(lib.dds_debug_read(self.ctx, what, module, index, slot, dev.data_ptr(), int(n), self._stream()))
        self.torch.cuda.synchronize(self.device)
        return dev.cpu().numpy()

    def dds_profile(self, enable):
        """0 / False: off; 1 / True: time launches on their concurrent streams; 2: modules serialised."""
        _check(lib.dds_profile(self.ctx, int(enable)))

    def dds_profile_read(self):
        """{class: (ms, launches, flops)}; classes forward / dgrad / wgrad on the generic kernels and
        forward_dma / dgrad_dma / wgrad_dma on the asynchronous global->LDS kernels."""
        out = (C.c_double * 18)()
        _check(lib.dds_profile_read(self.ctx, out))
        names = ("forward", "dgrad", "wgrad", "forward_dma", "dgrad_dma", "wgrad_dma")
        return {name: (out[3 * i], int(out[3 * i + 1]), out[3 * i + 2]) for i, name in enumerate(names)}

    def close(self):
        if getattr(self, "ctx", None):
            lib.dds_destroy(self.ctx)
            self.ctx = None
            self.arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
