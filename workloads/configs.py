"""Network descriptions and module splits for the five benchmark workloads.

A network is a list of blocks; a DDG run cuts that list into K consecutive
modules (Section 3 of the paper: the L layers are divided into K groups G(k)).
The residual architectures follow the paper's Table 2 (basic residual units,
widths 16-16-32-64, 9-9-9 units for ResNet-56 and 18-18-18 for ResNet-110);
ResNet-20 (3-3-3) and the bottleneck stage are the benchmark's additions.

Nothing here computes anything: only shapes, counts and names.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

BLOCK_STEM = 0        # conv3x3(cin->cout) + BN + ReLU
BLOCK_BASIC = 1       # conv3x3+BN+ReLU, conv3x3+BN, (+1x1 projection+BN), add, ReLU
BLOCK_BOTTLENECK = 2  # 1x1+BN+ReLU, 3x3+BN+ReLU, 1x1+BN, (+projection), add, ReLU
BLOCK_HEAD = 3        # global average pool + linear + softmax cross-entropy


@dataclass(frozen=True)
class Block:
    kind: int
    cin: int
    cmid: int
    cout: int
    stride: int = 1
    projection: int = 0

    def as_tuple(self) -> Tuple[int, int, int, int, int, int]:
        return (self.kind, self.cin, self.cmid, self.cout, self.stride,
                self.projection)


@dataclass
class ModuleSpec:
    """One module G(k): its blocks and the logical NCHW shape of its input."""
    k: int                      # 1-based
    blocks: List[Block]
    in_c: int
    in_h: int
    in_w: int
    out_c: int = 0
    out_h: int = 0
    out_w: int = 0


@dataclass
class Workload:
    name: str
    K: int
    batch: int
    num_classes: int            # 0 when the workload has no head
    modules: List[ModuleSpec]
    dtype: str                  # "f32" or "bf16": conv operand / activation type
    lr: float
    momentum: float
    weight_decay: float
    bn_eps: float
    steps: int                  # parity steps
    seed: int = 0
    notes: str = ""
    single_module: int = 0      # >0: only this module index is run (synthetic delta)


def conv_units(b: Block):
    """(name, cin, cout, ksize, stride) of each conv+BN unit, in parameter order."""
    if b.kind == BLOCK_STEM:
        return [("conv1", b.cin, b.cout, 3, b.stride)]
    if b.kind == BLOCK_BASIC:
        u = [("conv1", b.cin, b.cout, 3, b.stride), ("conv2", b.cout, b.cout, 3, 1)]
        if b.projection:
            u.append(("proj", b.cin, b.cout, 1, b.stride))
        return u
    if b.kind == BLOCK_BOTTLENECK:
        u = [("conv1", b.cin, b.cmid, 1, 1), ("conv2", b.cmid, b.cmid, 3, b.stride),
             ("conv3", b.cmid, b.cout, 1, 1)]
        if b.projection:
            u.append(("proj", b.cin, b.cout, 1, b.stride))
        return u
    return []


def block_param_shapes(b: Block, num_classes: int = 0):
    """Flat parameter order of one block: list of (name, shape).

    conv weights are [Cout][Cin][R][S]; each conv is followed by its BN scale
    and shift; the head holds fc.W [classes][C] then fc.b.
    """
    out = []
    if b.kind == BLOCK_HEAD:
        out.append(("fc.W", (num_classes, b.cin)))
        out.append(("fc.b", (num_classes,)))
        return out
    for name, ci, co, r, _ in conv_units(b):
        out.append((name + ".W", (co, ci, r, r)))
        out.append((name + ".bn.gamma", (co,)))
        out.append((name + ".bn.beta", (co,)))
    return out


def module_param_count(m: ModuleSpec, num_classes: int = 0) -> int:
    n = 0
    for b in m.blocks:
        for _, shp in block_param_shapes(b, num_classes):
            c = 1
            for d in shp:
                c *= d
            n += c
    return n


def _out_hw(h: int, stride: int) -> int:
    # 3x3 pad 1 and 1x1 pad 0 both give ceil(h / stride) for stride 1 and 2
    return (h - 1) // stride + 1


def _finish(mods: List[ModuleSpec]) -> None:
    for m in mods:
        c, h, w = m.in_c, m.in_h, m.in_w
        for b in m.blocks:
            if b.kind == BLOCK_HEAD:
                continue
            c, h, w = b.cout, _out_hw(h, b.stride), _out_hw(w, b.stride)
        m.out_c, m.out_h, m.out_w = c, h, w


def _split(blocks: List[Block], cuts: List[int], in_c: int, in_h: int, in_w: int):
    """Cut `blocks` before the indices in `cuts`; track each module's input shape."""
    bounds = [0] + list(cuts) + [len(blocks)]
    mods = []
    c, h, w = in_c, in_h, in_w
    for k in range(len(bounds) - 1):
        bl = blocks[bounds[k]:bounds[k + 1]]
        mods.append(ModuleSpec(k=k + 1, blocks=bl, in_c=c, in_h=h, in_w=w))
        for b in bl:
            if b.kind != BLOCK_HEAD:
                c, h, w = b.cout, _out_hw(h, b.stride), _out_hw(w, b.stride)
    _finish(mods)
    return mods


def cifar_resnet_blocks(units: int, num_classes: int, widths=(16, 32, 64)) -> List[Block]:
    """Stem + 3 groups of `units` basic blocks + head (Table 2 of the paper)."""
    blocks = [Block(BLOCK_STEM, 3, 0, widths[0], 1, 0)]
    cin = widths[0]
    for gi, wd in enumerate(widths):
        for u in range(units):
            stride = 2 if (gi > 0 and u == 0) else 1
            proj = 1 if (stride != 1 or cin != wd) else 0
            blocks.append(Block(BLOCK_BASIC, cin, 0, wd, stride, proj))
            cin = wd
    blocks.append(Block(BLOCK_HEAD, cin, 0, num_classes, 1, 0))
    return blocks


def _tiny() -> Workload:
    blocks = [Block(BLOCK_STEM, 3, 0, 16), Block(BLOCK_BASIC, 16, 0, 16),
              Block(BLOCK_BASIC, 16, 0, 16), Block(BLOCK_HEAD, 16, 0, 10)]
    mods = _split(blocks, [2], 3, 8, 8)
    return Workload("tiny_k2", 2, 4, 10, mods, "f32", 0.1, 0.9, 0.0, 1e-5, 5,
                    notes="stem + 2 basic blocks, 16 ch, 8x8, K=2")


def _resnet20() -> Workload:
    blocks = cifar_resnet_blocks(3, 10)
    # module 1 = stem + group 1 (blocks 0..3), module 2 = groups 2-3 + head
    mods = _split(blocks, [4], 3, 32, 32)
    return Workload("resnet20_k2", 2, 128, 10, mods, "f32", 0.01, 0.9, 0.0, 1e-5, 50,
                    notes="ResNet-20, split at the start of group 2")


def _resnet56() -> Workload:
    blocks = cifar_resnet_blocks(9, 10)
    mods = _split(blocks, [10, 19], 3, 32, 32)
    return Workload("resnet56_k3", 3, 128, 10, mods, "bf16", 0.01, 0.9, 0.0, 1e-5, 8,
                    notes="ResNet-56, K=3 at group boundaries")


def _resnet110() -> Workload:
    blocks = cifar_resnet_blocks(18, 100)
    # residual blocks 0-12 | 13-26 | 27-40 | 41-53 (+1 for the stem at index 0)
    mods = _split(blocks, [14, 28, 42], 3, 32, 32)
    return Workload("resnet110_k4", 4, 256, 100, mods, "bf16", 0.01, 0.9, 0.0, 1e-5, 8,
                    notes="ResNet-110, K=4, equal forward FLOPs at block boundaries")


def _bottleneck_slice(nblocks: int = 23, batch: int = 32, c: int = 1024, mid: int = 256,
                      hw: int = 14, name: str = "r101_stage3_k4m2") -> Workload:
    blocks = [Block(BLOCK_BOTTLENECK, c, mid, c, 1, 0) for _ in range(nblocks)]
    m = ModuleSpec(k=2, blocks=blocks, in_c=c, in_h=hw, in_w=hw)
    _finish([m])
    return Workload(name, 4, batch, 0, [m], "bf16", 0.01, 0.9, 0.0, 1e-5, 5,
                    notes="one module (k=2 of K=4) of bottleneck blocks, synthetic delta",
                    single_module=2)


def resnet8(split_layers=(3,), batch: int = 128, dtype: str = "f32", weight_decay: float = 0.0,
            lr: float = 1e-3) -> Workload:
    """ResNet-8 (Table 2: units 1-1-1, channels 16-16-32-64): stem = layer 1, three basic blocks
    = layers 2-3, 4-5, 6-7, classifier = layer 8. A split point "at layer l" (Section 5.1 uses
    1, 3, 5, 7, and 2 to 4 of them at once) cuts the network after layer l. Batch 128 and step
    size 1e-3 are Section 5.1's (Adam); synthetic CIFAR-10-shaped inputs."""
    for l in split_layers:
        if l not in (1, 3, 5, 7):
            raise ValueError("ResNet-8 split points lie after layers 1, 3, 5 or 7")
    blocks = cifar_resnet_blocks(1, 10)
    cuts = sorted((l + 1) // 2 for l in split_layers)
    mods = _split(blocks, cuts, 3, 32, 32)
    name = "resnet8_k%d_l%s" % (len(cuts) + 1, "".join(str(l) for l in sorted(split_layers)))
    return Workload(name, len(cuts) + 1, batch, 10, mods, dtype, lr, 0.9, weight_decay, 1e-5, 8,
                    notes="ResNet-8, split after layer(s) " + ",".join(str(l) for l in sorted(split_layers)))


WORKLOADS = {
    "tiny_k2": _tiny,
    "resnet20_k2": _resnet20,
    "resnet56_k3": _resnet56,
    "resnet110_k4": _resnet110,
    "r101_stage3_k4m2": _bottleneck_slice,
    # Section 5.1's network, one split point in the middle / four split points
    "resnet8_k2": lambda: resnet8((3,)),
    "resnet8_k5": lambda: resnet8((1, 3, 5, 7)),
}


def get_workload(name: str, **overrides) -> Workload:
    wl = WORKLOADS[name]()
    for key, val in overrides.items():
        setattr(wl, key, val)
    return wl


def custom_cifar(units: int, K_cuts: List[int], batch: int, num_classes: int, hw: int = 32,
                 dtype: str = "f32", widths=(16, 32, 64), name: str = "custom") -> Workload:
    """A CIFAR-style ResNet with arbitrary cut points (used by small parity cases)."""
    blocks = cifar_resnet_blocks(units, num_classes, widths)
    mods = _split(blocks, K_cuts, 3, hw, hw)
    return Workload(name, len(K_cuts) + 1, batch, num_classes, mods, dtype, 0.01, 0.9,
                    0.0, 1e-5, 5)


def custom_bottleneck(nblocks: int, batch: int, c: int, mid: int, hw: int,
                      K: int = 4, k: int = 2, name: str = "custom_bneck") -> Workload:
    wl = _bottleneck_slice(nblocks, batch, c, mid, hw, name)
    wl.K = K
    wl.modules[0].k = k
    wl.single_module = k
    return wl
