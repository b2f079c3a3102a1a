"""Seeded initial weights, minibatches and synthetic error gradients.

All arrays are float64 in logical NCHW / [Cout][Cin][R][S] order; callers cast
and re-lay them out for whichever implementation they feed.
"""
from __future__ import annotations

import numpy as np

from .configs import Workload, ModuleSpec, block_param_shapes
from .rng import normal, uniform_int


def init_module_params(wl: Workload, m: ModuleSpec, perturb_bn: bool = False) -> np.ndarray:
    """Flat parameter vector of module m in the boundary's parameter order.

    conv W ~ N(0, 2/(Cin*R*S)) (He-normal, fan-in); BN gamma=1, beta=0
    (or gamma=1+0.1n, beta=0.1n when perturb_bn, to make tests sensitive to
    the BN parameters); fc.W ~ N(0, 1/C), fc.b = 0.
    """
    parts = []
    ti = 0
    for bi, b in enumerate(m.blocks):
        for name, shp in block_param_shapes(b, wl.num_classes):
            n = int(np.prod(shp))
            stream = 10_000 * m.k + 100 * bi + ti % 100
            ti += 1
            if name.endswith(".W") and len(shp) == 4:
                fan_in = shp[1] * shp[2] * shp[3]
                v = normal(wl.seed, stream, n) * np.sqrt(2.0 / fan_in)
            elif name == "fc.W":
                v = normal(wl.seed, stream, n) * np.sqrt(1.0 / shp[1])
            elif name.endswith("gamma"):
                v = np.ones(n)
                if perturb_bn:
                    v = v + 0.1 * normal(wl.seed, stream, n)
            else:  # beta, fc.b
                v = np.zeros(n)
                if perturb_bn:
                    v = v + 0.1 * normal(wl.seed, stream, n)
            parts.append(v)
    return np.concatenate(parts) if parts else np.zeros(0)


def minibatch(wl: Workload, t: int):
    """Minibatch t of the full network: x [N,3,H,W] ~ N(0,1), labels uniform."""
    m0 = wl.modules[0]
    n = wl.batch * m0.in_c * m0.in_h * m0.in_w
    x = normal(wl.seed, 1_000_000 + t, n).reshape(wl.batch, m0.in_c, m0.in_h, m0.in_w)
    classes = max(wl.num_classes, 1)
    y = uniform_int(wl.seed, 2_000_000 + t, wl.batch, classes)
    return x, y


def synthetic_delta(wl: Workload, m: ModuleSpec, t: int, sigma: float = 1e-2) -> np.ndarray:
    """A stand-in error gradient for a module with no real producer: N(0, sigma^2)."""
    n = wl.batch * m.out_c * m.out_h * m.out_w
    return (sigma * normal(wl.seed, 3_000_000 + t, n)).reshape(wl.batch, m.out_c, m.out_h, m.out_w)
