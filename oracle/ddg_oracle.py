"""ctypes binding of the CPU oracle (oracle/ddg_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
bench's cpu_baseline leg. The HIP library and its Python binding never import
this module.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ddg_oracle.cpp")
_LIB = os.path.join(_HERE, "libddg_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (OpenMP over independent output slices only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O3", "-fopenmp", "-std=c++17", "-shared", "-fPIC",
                               "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        for sfx in ("f64", "f32"):
            getattr(_lib, f"orc_create_{sfx}").restype = C.c_void_p
            for n in ("param_count", "in_size", "out_size", "get_delta", "fifo_depth", "time", "get_updates", "running_count"):
                getattr(_lib, f"orc_{n}_{sfx}").restype = C.c_long
            for n in ("head", "ddg_step", "bp_step"):
                getattr(_lib, f"orc_{n}_{sfx}").restype = C.c_double
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


class _Typed:
    def __init__(self, dtype):
        self.np = np.float64 if dtype in ("f64", np.float64) else np.float32
        self.sfx = "f64" if self.np is np.float64 else "f32"

    def fn(self, name):
        return getattr(lib(), f"orc_{name}_{self.sfx}")

    def arr(self, a):
        return np.ascontiguousarray(a, dtype=self.np)


# --- single layers (NCHW, [Cout][Cin][R][S]) ---------------------------------------

def conv_fwd(x, w, stride=1, pad=None, dtype="f64"):
    ty = _Typed(dtype)
    x, w = ty.arr(x), ty.arr(w)
    N, Ci, H, W = x.shape
    Co, _, R, _ = w.shape
    pad = (1 if R == 3 else 0) if pad is None else pad
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    y = np.empty((N, Co, P, Q), ty.np)
    ty.fn("conv_fwd")(_p(x), _p(w), _p(y), N, Ci, H, W, Co, R, stride, pad)
    return y


def conv_bwd_data(dy, w, in_hw, stride=1, pad=None, dtype="f64"):
    ty = _Typed(dtype)
    dy, w = ty.arr(dy), ty.arr(w)
    N, Co, _, _ = dy.shape
    _, Ci, R, _ = w.shape
    H, W = in_hw
    pad = (1 if R == 3 else 0) if pad is None else pad
    dx = np.empty((N, Ci, H, W), ty.np)
    ty.fn("conv_bwd_data")(_p(dy), _p(w), _p(dx), N, Ci, H, W, Co, R, stride, pad)
    return dx


def conv_bwd_weight(x, dy, R, stride=1, pad=None, dtype="f64"):
    ty = _Typed(dtype)
    x, dy = ty.arr(x), ty.arr(dy)
    N, Ci, H, W = x.shape
    Co = dy.shape[1]
    pad = (1 if R == 3 else 0) if pad is None else pad
    dw = np.empty((Co, Ci, R, R), ty.np)
    ty.fn("conv_bwd_weight")(_p(x), _p(dy), _p(dw), N, Ci, H, W, Co, R, stride, pad)
    return dw


def bn_fwd(x, gamma, beta, eps=1e-5, dtype="f64"):
    ty = _Typed(dtype)
    x, gamma, beta = ty.arr(x), ty.arr(gamma), ty.arr(beta)
    N, Cc, H, W = x.shape
    y = np.empty_like(x)
    mean, invstd = np.empty(Cc, ty.np), np.empty(Cc, ty.np)
    ty.fn("bn_fwd")(_p(x), _p(gamma), _p(beta), C.c_double(eps), _p(y), _p(mean), _p(invstd),
                    N, Cc, H * W)
    return y, mean, invstd


def bn_bwd(dy, x, mean, invstd, gamma, dtype="f64"):
    ty = _Typed(dtype)
    dy, x, mean, invstd, gamma = map(ty.arr, (dy, x, mean, invstd, gamma))
    N, Cc, H, W = x.shape
    dx = np.empty_like(x)
    dg, db = np.empty(Cc, ty.np), np.empty(Cc, ty.np)
    ty.fn("bn_bwd")(_p(dy), _p(x), _p(mean), _p(invstd), _p(gamma), _p(dx), _p(dg), _p(db),
                    N, Cc, H * W)
    return dx, dg, db


def head(h, fcw, fcb, labels, want_grads=True, dtype="f64"):
    ty = _Typed(dtype)
    h, fcw, fcb = ty.arr(h), ty.arr(fcw), ty.arr(fcb)
    labels = np.ascontiguousarray(labels, np.int32)
    N, Cc, H, W = h.shape
    classes = fcw.shape[0]
    logits = np.empty((N, classes), ty.np)
    dh = np.empty_like(h) if want_grads else None
    dw = np.empty_like(fcw) if want_grads else None
    db = np.empty_like(fcb) if want_grads else None
    loss = ty.fn("head")(_p(h), _p(fcw), _p(fcb), _p(labels), N, Cc, H * W, classes,
                         _p(dh), _p(dw), _p(db), _p(logits))
    return float(loss), logits, dh, dw, db


def round_bf16(a, dtype="f64"):
    """Round to bfloat16 (nearest-even) and return in the oracle's scalar type."""
    ty = _Typed(dtype)
    v = ty.arr(a).copy()
    ty.fn("round_bf16")(_p(v), C.c_long(v.size))
    return v


# --- whole networks -----------------------------------------------------------------

class OracleNet:
    """K modules (or a single module k of K) with FIFOs, inboxes and momentum SGD.

    `modules` is a list of (in-order) block lists; each block is a 6-tuple
    (kind, cin, cmid, cout, stride, projection).
    """

    def __init__(self, K, modules, batch, in_chw, num_classes, momentum=0.9, weight_decay=0.0,
                 bn_eps=1e-5, dtype="f64", stale_jacobian=False, k_first=1, store_bf16=False):
        self.ty = _Typed(dtype)
        self.K, self.k_first, self.nmods = K, k_first, len(modules)
        self.batch = batch
        self.num_classes = num_classes
        self._has_head = [any(b[0] == 3 for b in m) for m in modules]   # block kind 3: the classifier
        nblocks = np.array([len(m) for m in modules], np.int32)
        desc = np.array([v for m in modules for b in m for v in b], np.int32)
        self._h = C.c_void_p(self.ty.fn("create")(
            K, k_first, self.nmods, _p(nblocks), _p(desc), batch, in_chw[0], in_chw[1], in_chw[2],
            num_classes, C.c_double(momentum), C.c_double(weight_decay), C.c_double(bn_eps),
            1 if stale_jacobian else 0, 1 if store_bf16 else 0))

    @classmethod
    def from_workload(cls, wl, dtype="f64", stale_jacobian=False, batch=None, store_bf16=None):
        """store_bf16 defaults to the workload's storage type (bf16 workloads round stored tensors)."""
        if store_bf16 is None:
            store_bf16 = (wl.dtype == "bf16")
        mods = [[b.as_tuple() for b in m.blocks] for m in wl.modules]
        m0 = wl.modules[0]
        return cls(wl.K, mods, batch or wl.batch, (m0.in_c, m0.in_h, m0.in_w), wl.num_classes,
                   wl.momentum, wl.weight_decay, wl.bn_eps, dtype, stale_jacobian, k_first=m0.k,
                   store_bf16=store_bf16)

    def __del__(self):
        try:
            self.ty.fn("destroy")(self._h)
        except Exception:
            pass

    def ks(self):
        return range(self.k_first, self.k_first + self.nmods)

    def param_count(self, k):
        return int(self.ty.fn("param_count")(self._h, k))

    def out_shape(self, k):
        chw = np.zeros(3, np.int32)
        self.ty.fn("out_shape")(self._h, k, _p(chw))
        return (self.batch, int(chw[0]), int(chw[1]), int(chw[2]))

    def in_size(self, k):
        return int(self.ty.fn("in_size")(self._h, k))

    def set_params(self, k, v):
        v = self.ty.arr(v)
        assert v.size == self.param_count(k)
        self.ty.fn("set_params")(self._h, k, _p(v))

    def set_velocity(self, k, v):
        v = self.ty.arr(v)
        assert v.size == self.param_count(k)
        self.ty.fn("set_velocity")(self._h, k, _p(v))

    def _get(self, name, k):
        v = np.empty(self.param_count(k), self.ty.np)
        r = self.ty.fn(name)(self._h, k, _p(v))
        return v, r

    def get_params(self, k):
        return self._get("get_params", k)[0]

    def get_velocity(self, k):
        return self._get("get_velocity", k)[0]

    def get_grad(self, k):
        v, valid = self._get("get_grad", k)
        return v if valid else None

    def get_h(self, k):
        v = np.empty(self.out_shape(k), self.ty.np)
        self.ty.fn("get_h")(self._h, k, _p(v))
        return v

    def get_delta(self, k):
        """(delta at module k's output, iteration it belongs to) or (None, -1)."""
        v = np.empty(self.out_shape(k), self.ty.np)
        ts = int(self.ty.fn("get_delta")(self._h, k, _p(v)))
        return (v, ts) if ts >= 0 else (None, -1)

    def get_logits(self, k, classes):
        v = np.empty((self.batch, classes), self.ty.np)
        self.ty.fn("get_logits")(self._h, k, _p(v))
        return v

    def fifo_depth(self, k):
        return int(self.ty.fn("fifo_depth")(self._h, k))

    def time(self):
        return int(self.ty.fn("time")(self._h))

    # module-level calls (mirror the boundary of the HIP library)
    def forward(self, k, t, h_in):
        h_in = self.ty.arr(h_in)
        assert h_in.size == self.in_size(k)
        out = np.empty(self.out_shape(k), self.ty.np)
        self.ty.fn("forward")(self._h, k, C.c_long(t), _p(h_in), _p(out))
        return out

    def backward_delayed(self, k, t, delta_in=None, labels=None, in_shape=None):
        """Returns (did_backward, delta_out or None, loss or None)."""
        din = self.ty.arr(delta_in) if delta_in is not None else None
        lab = np.ascontiguousarray(labels, np.int32) if labels is not None else None
        dout = np.zeros(self.in_size(k), self.ty.np)
        loss = np.zeros(1, self.ty.np)
        did = int(self.ty.fn("backward_delayed")(self._h, k, C.c_long(t), _p(din), _p(lab),
                                                 _p(dout), _p(loss)))
        if in_shape is not None:
            dout = dout.reshape(in_shape)
        return did, (dout if k > 1 else None), float(loss[0])

    def update(self, k, lr):
        self.ty.fn("update")(self._h, k, C.c_double(lr))

    # evaluation: running BN estimates (per conv unit in parameter order: mean[C], variance[C])
    def set_bn_momentum(self, rho):
        self.ty.fn("set_bn_momentum")(self._h, C.c_double(rho))

    def running_count(self, k):
        return int(self.ty.fn("running_count")(self._h, k))

    def get_running(self, k):
        v = np.empty(self.running_count(k), self.ty.np)
        self.ty.fn("get_running")(self._h, k, _p(v))
        return v

    def set_running(self, k, v):
        v = self.ty.arr(v)
        assert v.size == self.running_count(k)
        self.ty.fn("set_running")(self._h, k, _p(v))

    def forward_eval(self, k, h_in, labels=None):
        """Evaluation forward of module k. Without a head: the module output. With a head:
        (mean loss or None without labels, logits[N, classes])."""
        h_in = self.ty.arr(h_in)
        assert h_in.size == self.in_size(k)
        if not self._has_head[k - self.k_first]:
            out = np.empty(self.out_shape(k), self.ty.np)
            self.ty.fn("forward_eval")(self._h, k, _p(h_in), _p(out), None, None, None)
            return out
        lab = np.ascontiguousarray(labels, np.int32) if labels is not None else None
        loss = np.zeros(1, self.ty.np)
        logits = np.empty((self.batch, self.num_classes), self.ty.np)
        self.ty.fn("forward_eval")(self._h, k, _p(h_in), None, _p(lab), _p(loss), _p(logits))
        return (float(loss[0]) if labels is not None else None), logits

    # Adam with delayed gradients (Algorithm 2) instead of momentum SGD
    def set_adam(self, on=True, beta1=0.9, beta2=0.999, eps=1e-8):
        self.ty.fn("set_adam")(self._h, int(on), C.c_double(beta1), C.c_double(beta2), C.c_double(eps))

    def get_moment2(self, k):
        return self._get("get_moment2", k)[0]

    def set_moment2(self, k, v):
        v = self.ty.arr(v)
        assert v.size == self.param_count(k)
        self.ty.fn("set_moment2")(self._h, k, _p(v))

    def get_updates(self, k) -> int:
        return int(self.ty.fn("get_updates")(self._h, k))

    def set_updates(self, k, n):
        self.ty.fn("set_updates")(self._h, k, C.c_long(n))

    # drivers
    def ddg_step(self, x, labels, lr):
        x = self.ty.arr(x)
        labels = np.ascontiguousarray(labels, np.int32)
        return float(self.ty.fn("ddg_step")(self._h, _p(x), _p(labels), C.c_double(lr)))

    def bp_step(self, x, labels, lr, update=True):
        x = self.ty.arr(x)
        labels = np.ascontiguousarray(labels, np.int32)
        return float(self.ty.fn("bp_step")(self._h, _p(x), _p(labels), C.c_double(lr),
                                           1 if update else 0))
