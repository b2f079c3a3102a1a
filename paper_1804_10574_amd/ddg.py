"""ctypes binding of libddg.so: same names as include/ddg.h, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

DDG_F32, DDG_BF16 = 0, 1
DDG_OPT_SGD, DDG_OPT_ADAM = 0, 1
_STATUS = {0: "DDG_OK", 1: "DDG_ERR_INVALID_ARG", 2: "DDG_ERR_SHAPE", 3: "DDG_ERR_STATE",
           4: "DDG_ERR_OOM", 5: "DDG_ERR_DEVICE"}

_HERE = os.path.dirname(os.path.abspath(__file__))


def library_path() -> str:
    return os.path.join(_HERE, "libddg.so")


class DDGError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{_STATUS.get(status, status)}: {msg}")
        self.status = status


class BlockDesc(C.Structure):
    _fields_ = [("kind", C.c_int), ("cin", C.c_int), ("cmid", C.c_int), ("cout", C.c_int),
                ("stride", C.c_int), ("projection", C.c_int)]


class ModuleDesc(C.Structure):
    _fields_ = [("K", C.c_int), ("k", C.c_int), ("batch", C.c_int), ("in_c", C.c_int),
                ("in_h", C.c_int), ("in_w", C.c_int), ("num_blocks", C.c_int),
                ("blocks", C.POINTER(BlockDesc)), ("num_classes", C.c_int), ("compute", C.c_int),
                ("momentum", C.c_float), ("weight_decay", C.c_float), ("bn_eps", C.c_float),
                ("stream", C.c_void_p), ("forward_stream", C.c_void_p), ("dry_run", C.c_int),
                ("stale_jacobian", C.c_int)]


_lib = None


def load_library():
    """Load libddg.so built in-tree (python -m paper_1804_10574_amd.build). Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} is missing: build it first (python paper_1804_10574_amd/build.py). "
            "There is no CPU fallback.")
    lib = C.CDLL(path)
    vp, st = C.c_void_p, C.c_int
    sig = {
        "ddg_module_create": (st, [C.POINTER(ModuleDesc), C.POINTER(vp)]),
        "ddg_module_destroy": (st, [vp]),
        "ddg_param_count": (C.c_size_t, [vp]),
        "ddg_out_shape": (st, [vp, C.POINTER(C.c_int), C.POINTER(C.c_int), C.POINTER(C.c_int)]),
        "ddg_device_bytes": (C.c_size_t, [vp]),
        "ddg_set_params": (st, [vp, vp, C.c_int]),
        "ddg_set_velocity": (st, [vp, vp, C.c_int]),
        "ddg_get_params": (st, [vp, vp]),
        "ddg_get_velocity": (st, [vp, vp]),
        "ddg_get_grad": (st, [vp, vp, C.POINTER(C.c_int)]),
        "ddg_forward": (st, [vp, C.c_long, vp, vp]),
        "ddg_backward_delayed": (st, [vp, C.c_long, vp, vp, vp, vp, C.POINTER(C.c_int)]),
        "ddg_update": (st, [vp, C.c_long, C.c_float]),
        "ddg_set_optimizer": (st, [vp, C.c_int, C.c_float, C.c_float, C.c_float]),
        "ddg_set_moment2": (st, [vp, vp, C.c_int]),
        "ddg_get_moment2": (st, [vp, vp]),
        "ddg_set_update_count": (st, [vp, C.c_long]),
        "ddg_get_update_count": (C.c_long, [vp]),
        "ddg_pipeline_set_optimizer": (st, [vp, C.c_int, C.c_float, C.c_float, C.c_float]),
        "ddg_set_bn_momentum": (st, [vp, C.c_float]),
        "ddg_running_count": (C.c_size_t, [vp]),
        "ddg_get_running": (st, [vp, vp]),
        "ddg_set_running": (st, [vp, vp]),
        "ddg_forward_eval": (st, [vp, vp, vp, vp, vp, vp]),
        "ddg_forward_eval_static": (st, [vp, vp, vp, vp, vp, vp]),
        "ddg_pipeline_forward_eval": (st, [vp, vp, vp, vp, vp]),
        "ddg_pipeline_set_bn_momentum": (st, [vp, C.c_float]),
        "ddg_module_sync": (st, [vp]),
        "ddg_ring_slots": (C.c_int, [vp]),
        "ddg_ring_slot_bytes": (C.c_size_t, [vp]),
        "ddg_get_ring_slot": (st, [vp, C.c_int, vp]),
        "ddg_set_ring_slot": (st, [vp, C.c_int, vp]),
        "ddg_set_time": (st, [vp, C.c_long]),
        "ddg_get_time": (C.c_long, [vp]),
        "ddg_pipeline_time": (C.c_long, [vp]),
        "ddg_pipeline_set_time": (st, [vp, C.c_long]),
        "ddg_pipeline_mail_bytes": (C.c_size_t, [vp, C.c_int]),
        "ddg_pipeline_get_mail": (st, [vp, C.c_int, vp, C.POINTER(C.c_long)]),
        "ddg_pipeline_set_mail": (st, [vp, C.c_int, vp, C.c_long]),
        "ddg_pipeline_create": (st, [C.POINTER(ModuleDesc), C.c_int, C.POINTER(vp), C.POINTER(vp)]),
        "ddg_pipeline_destroy": (st, [vp]),
        "ddg_pipeline_module": (vp, [vp, C.c_int]),
        "ddg_pipeline_step": (st, [vp, vp, vp, C.c_float, vp]),
        "ddg_pipeline_set_graphs": (st, [vp, C.c_int]),
        "ddg_pipeline_get_h": (st, [vp, C.c_int, vp]),
        "ddg_pipeline_get_delta": (st, [vp, C.c_int, vp, C.POINTER(C.c_long)]),
        "ddg_pipeline_sync": (st, [vp]),
        "ddg_profile_kinds": (C.c_int, []),
        "ddg_profile_kind_name": (C.c_char_p, [C.c_int]),
        "ddg_profile_enable": (st, [vp, C.c_int]),
        "ddg_profile_read": (st, [vp, C.c_int, C.POINTER(C.c_long), C.POINTER(C.c_double),
                                  C.POINTER(C.c_double), C.POINTER(C.c_double)]),
        "ddg_profile_reset": (st, [vp]),
        "ddg_last_error": (C.c_char_p, []),
        "ddg_version": (C.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


EXPORTS = ["ddg_module_create", "ddg_module_destroy", "ddg_param_count", "ddg_out_shape",
           "ddg_device_bytes", "ddg_set_params", "ddg_set_velocity", "ddg_get_params", "ddg_get_velocity", "ddg_get_grad",
           "ddg_forward", "ddg_backward_delayed", "ddg_update", "ddg_module_sync",
           "ddg_set_optimizer", "ddg_set_moment2", "ddg_get_moment2", "ddg_set_update_count", "ddg_get_update_count",
           "ddg_pipeline_set_optimizer",
           "ddg_set_bn_momentum", "ddg_running_count", "ddg_get_running", "ddg_set_running", "ddg_forward_eval", "ddg_forward_eval_static",
           "ddg_pipeline_forward_eval", "ddg_pipeline_set_bn_momentum",
           "ddg_pipeline_create", "ddg_pipeline_destroy", "ddg_pipeline_module", "ddg_pipeline_step",
           "ddg_pipeline_set_graphs", "ddg_pipeline_get_h", "ddg_pipeline_get_delta", "ddg_pipeline_sync", "ddg_profile_kinds",
           "ddg_profile_kind_name", "ddg_profile_enable", "ddg_profile_read", "ddg_profile_reset",
           "ddg_ring_slots", "ddg_ring_slot_bytes", "ddg_get_ring_slot", "ddg_set_ring_slot", "ddg_set_time", "ddg_get_time",
           "ddg_pipeline_time", "ddg_pipeline_set_time", "ddg_pipeline_mail_bytes", "ddg_pipeline_get_mail",
           "ddg_pipeline_set_mail",
           "ddg_last_error", "ddg_version"]


def _check(status: int):
    if status != 0:
        raise DDGError(status, load_library().ddg_last_error().decode())


def version() -> str:
    return load_library().ddg_version().decode()


def profile_kinds() -> List[str]:
    lib = load_library()
    return [lib.ddg_profile_kind_name(i).decode() for i in range(lib.ddg_profile_kinds())]


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return t.ctypes.data


def make_desc(K, k, batch, in_chw, blocks: Sequence[Sequence[int]], num_classes, compute, momentum,
              weight_decay, bn_eps, stream=None, dry_run=False, forward_stream=None, stale_jacobian=False):
    arr = (BlockDesc * len(blocks))(*[BlockDesc(*b) for b in blocks])
    d = ModuleDesc(K, k, batch, in_chw[0], in_chw[1], in_chw[2], len(blocks), arr, num_classes,
                   compute, momentum, weight_decay, bn_eps, stream, forward_stream, 1 if dry_run else 0,
                   1 if stale_jacobian else 0)
    d._keep = arr
    return d


class Module:
    """One module G(k): ddg_forward / ddg_backward_delayed / ddg_update."""

    def __init__(self, desc: ModuleDesc = None, handle=None, owner=None):
        self._lib = load_library()
        self._owner = owner
        if handle is not None:
            self._h = C.c_void_p(handle)
            return
        h = C.c_void_p()
        _check(self._lib.ddg_module_create(C.byref(desc), C.byref(h)))
        self._h = h

    def close(self):
        if self._owner is None and self._h:
            self._lib.ddg_module_destroy(self._h)
        self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def param_count(self) -> int:
        return int(self._lib.ddg_param_count(self._h))

    def device_bytes(self) -> int:
        return int(self._lib.ddg_device_bytes(self._h))

    def out_shape(self):
        c, h, w = C.c_int(), C.c_int(), C.c_int()
        _check(self._lib.ddg_out_shape(self._h, C.byref(c), C.byref(h), C.byref(w)))
        return c.value, h.value, w.value

    def set_params(self, src, is_device=False):
        if not is_device:
            src = np.ascontiguousarray(src, np.float32)
            assert src.size == self.param_count()
        _check(self._lib.ddg_set_params(self._h, _ptr(src), 1 if is_device else 0))

    def set_velocity(self, src, is_device=False):
        if not is_device:
            src = np.ascontiguousarray(src, np.float32)
            assert src.size == self.param_count()
        _check(self._lib.ddg_set_velocity(self._h, _ptr(src), 1 if is_device else 0))

    def set_optimizer(self, kind, beta1=0.9, beta2=0.999, eps=1e-8):
        _check(self._lib.ddg_set_optimizer(self._h, kind, beta1, beta2, eps))

    def set_moment2(self, src, is_device=False):
        if not is_device:
            src = np.ascontiguousarray(src, np.float32)
            assert src.size == self.param_count()
        _check(self._lib.ddg_set_moment2(self._h, _ptr(src), 1 if is_device else 0))

    def get_moment2(self):
        out, st = self._get(self._lib.ddg_get_moment2)
        _check(st)
        return out

    def set_update_count(self, n):
        _check(self._lib.ddg_set_update_count(self._h, n))

    def get_update_count(self) -> int:
        return int(self._lib.ddg_get_update_count(self._h))

    def _get(self, fn):
        out = np.empty(self.param_count(), np.float32)
        return out, fn(self._h, _ptr(out))

    # evaluation: running BN estimates (per conv unit in parameter order: mean[C], variance[C])
    def set_bn_momentum(self, rho):
        _check(self._lib.ddg_set_bn_momentum(self._h, rho))

    def running_count(self) -> int:
        return int(self._lib.ddg_running_count(self._h))

    def get_running(self):
        out = np.empty(self.running_count(), np.float32)
        _check(self._lib.ddg_get_running(self._h, _ptr(out)))
        return out

    def set_running(self, src):
        src = np.ascontiguousarray(src, np.float32)
        assert src.size == self.running_count()
        _check(self._lib.ddg_set_running(self._h, _ptr(src)))

    def forward_eval(self, h_in, h_out=None, labels=None, loss_out=None, logits_out=None):
        _check(self._lib.ddg_forward_eval(self._h, _ptr(h_in), _ptr(h_out), _ptr(labels), _ptr(loss_out),
                                          _ptr(logits_out)))

    def forward_eval_static(self, h_in, h_out=None, labels=None, loss_out=None, logits_out=None):
        _check(self._lib.ddg_forward_eval_static(self._h, _ptr(h_in), _ptr(h_out), _ptr(labels), _ptr(loss_out),
                                                 _ptr(logits_out)))

    def get_params(self):
        out = np.empty(self.param_count(), np.float32)
        _check(self._lib.ddg_get_params(self._h, _ptr(out)))
        return out

    def get_velocity(self):
        out = np.empty(self.param_count(), np.float32)
        _check(self._lib.ddg_get_velocity(self._h, _ptr(out)))
        return out

    def get_grad(self):
        out = np.empty(self.param_count(), np.float32)
        valid = C.c_int()
        _check(self._lib.ddg_get_grad(self._h, _ptr(out), C.byref(valid)))
        return out if valid.value else None

    def forward(self, t, h_in, h_out):
        _check(self._lib.ddg_forward(self._h, t, _ptr(h_in), _ptr(h_out)))

    def backward_delayed(self, t, delta_in=None, labels=None, delta_out=None, loss_out=None) -> bool:
        did = C.c_int()
        _check(self._lib.ddg_backward_delayed(self._h, t, _ptr(delta_in), _ptr(labels), _ptr(delta_out),
                                              _ptr(loss_out), C.byref(did)))
        return bool(did.value)

    def update(self, t, lr):
        _check(self._lib.ddg_update(self._h, t, lr))

    def sync(self):
        _check(self._lib.ddg_module_sync(self._h))

    # checkpoint of the delay ring: raw slots (bytes of the compute type) and the iteration counter
    def ring_slots(self) -> int:
        return int(self._lib.ddg_ring_slots(self._h))

    def get_ring_slot(self, slot):
        out = np.empty(int(self._lib.ddg_ring_slot_bytes(self._h)), np.uint8)
        _check(self._lib.ddg_get_ring_slot(self._h, slot, _ptr(out)))
        return out

    def set_ring_slot(self, slot, src):
        src = np.ascontiguousarray(src, np.uint8)
        assert src.size == int(self._lib.ddg_ring_slot_bytes(self._h))
        _check(self._lib.ddg_set_ring_slot(self._h, slot, _ptr(src)))

    def set_time(self, t):
        _check(self._lib.ddg_set_time(self._h, t))

    def get_time(self) -> int:
        return int(self._lib.ddg_get_time(self._h))

    def profile_enable(self, on=True):
        _check(self._lib.ddg_profile_enable(self._h, 1 if on else 0))

    def profile_reset(self):
        _check(self._lib.ddg_profile_reset(self._h))

    def profile_read(self):
        """-> {kind name: (launches, total_ms, algorithmic bytes, algorithmic flops)}"""
        out = {}
        for i, name in enumerate(profile_kinds()):
            n, ms, nb, fl = C.c_long(), C.c_double(), C.c_double(), C.c_double()
            _check(self._lib.ddg_profile_read(self._h, i, C.byref(n), C.byref(ms), C.byref(nb), C.byref(fl)))
            out[name] = (n.value, ms.value, nb.value, fl.value)
        return out


class Pipeline:
    """K modules as concurrent streams: ddg_pipeline_*."""

    def __init__(self, descs: Sequence[ModuleDesc], streams: Optional[Sequence[int]] = None):
        self._lib = load_library()
        K = len(descs)
        arr = (ModuleDesc * K)(*descs)
        self._keep = (arr, list(descs))
        sp = None
        if streams is not None:
            sp = (C.c_void_p * K)(*[C.c_void_p(s) for s in streams])
        h = C.c_void_p()
        _check(self._lib.ddg_pipeline_create(arr, K, sp, C.byref(h)))
        self._h = h
        self.K = K
        self.batch = descs[0].batch

    def close(self):
        if self._h:
            self._lib.ddg_pipeline_destroy(self._h)
        self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def module(self, k) -> Module:
        return Module(handle=self._lib.ddg_pipeline_module(self._h, k), owner=self)

    def step(self, x, labels, lr, loss_out=None):
        _check(self._lib.ddg_pipeline_step(self._h, _ptr(x), _ptr(labels), lr, _ptr(loss_out)))

    def set_graphs(self, on: bool):
        _check(self._lib.ddg_pipeline_set_graphs(self._h, 1 if on else 0))

    def set_optimizer(self, kind, beta1=0.9, beta2=0.999, eps=1e-8):
        _check(self._lib.ddg_pipeline_set_optimizer(self._h, kind, beta1, beta2, eps))

    def set_bn_momentum(self, rho):
        _check(self._lib.ddg_pipeline_set_bn_momentum(self._h, rho))

    def forward_eval(self, x, labels=None, loss_out=None, logits_out=None):
        _check(self._lib.ddg_pipeline_forward_eval(self._h, _ptr(x), _ptr(labels), _ptr(loss_out), _ptr(logits_out)))

    def sync(self):
        _check(self._lib.ddg_pipeline_sync(self._h))

    # checkpoint of the pipeline's own state: the iteration counter and the error gradients in flight
    def time(self) -> int:
        return int(self._lib.ddg_pipeline_time(self._h))

    def set_time(self, t):
        _check(self._lib.ddg_pipeline_set_time(self._h, t))

    def get_mail(self, k):
        """-> (raw bytes of the gradient in flight to module k, its iteration), or (None, -1)."""
        out = np.empty(int(self._lib.ddg_pipeline_mail_bytes(self._h, k)), np.uint8)
        it = C.c_long()
        _check(self._lib.ddg_pipeline_get_mail(self._h, k, _ptr(out), C.byref(it)))
        return (out, it.value) if it.value >= 0 else (None, -1)

    def set_mail(self, k, src, iteration):
        src = np.ascontiguousarray(src, np.uint8)
        assert src.size == int(self._lib.ddg_pipeline_mail_bytes(self._h, k))
        _check(self._lib.ddg_pipeline_set_mail(self._h, k, _ptr(src), iteration))

    def get_h(self, k):
        c, h, w = self.module(k).out_shape()
        out = np.empty((self.batch, h, w, c), np.float32)
        _check(self._lib.ddg_pipeline_get_h(self._h, k, _ptr(out)))
        return out

    def get_delta(self, k):
        c, h, w = self.module(k).out_shape()
        out = np.empty((self.batch, h, w, c), np.float32)
        it = C.c_long()
        _check(self._lib.ddg_pipeline_get_delta(self._h, k, _ptr(out), C.byref(it)))
        return (out, it.value) if it.value >= 0 else (None, -1)
