"""Independent comparator for tests: the same networks built from CPU PyTorch
float64 library ops with autograd. Test-only; neither the oracle nor the HIP
library uses it."""
import numpy as np
import torch
import torch.nn.functional as F

from workloads import BLOCK_STEM, BLOCK_BASIC, BLOCK_BOTTLENECK, BLOCK_HEAD, block_param_shapes


def unflatten(blocks, flat, num_classes):
    """-> list (per block) of dict name -> torch tensor (requires_grad)."""
    out, off = [], 0
    for b in blocks:
        d = {}
        for name, shp in block_param_shapes(b, num_classes):
            n = int(np.prod(shp))
            d[name] = torch.tensor(np.asarray(flat[off:off + n], np.float64).reshape(shp),
                                   dtype=torch.float64, requires_grad=True)
            off += n
        out.append(d)
    assert off == len(flat)
    return out


def flatten_grads(params):
    return np.concatenate([p.grad.numpy().ravel() if p.grad is not None else np.zeros(p.numel())
                           for d in params for p in d.values()])


def unit_names(b):
    """Conv units of a block in parameter order."""
    if b.kind == BLOCK_HEAD:
        return []
    names = {BLOCK_STEM: ["conv1"], BLOCK_BASIC: ["conv1", "conv2"], BLOCK_BOTTLENECK: ["conv1", "conv2", "conv3"]}[b.kind]
    return names + (["proj"] if b.projection and b.kind != BLOCK_STEM else [])


def new_running(blocks, params):
    """Running BN estimates in the library's starting state: per block a dict name -> [mean, var]."""
    return [{n: [torch.zeros(p[n + ".W"].shape[0], dtype=torch.float64), torch.ones(p[n + ".W"].shape[0], dtype=torch.float64)]
             for n in unit_names(b)} for b, p in zip(blocks, params)]


def flatten_running(blocks, running):
    """The flat layout of the oracle and the library: per conv unit mean[C], then variance[C]."""
    return np.concatenate([t.numpy().ravel() for b, r in zip(blocks, running) for n in unit_names(b) for t in r[n]])


def _unit(x, p, name, stride, eps, run=None, training=True, momentum=0.1):
    w = p[name + ".W"]
    pad = 1 if w.shape[-1] == 3 else 0
    z = F.conv2d(x, w, stride=stride, padding=pad)
    if run is None:
        return F.batch_norm(z, None, None, p[name + ".bn.gamma"], p[name + ".bn.beta"], True, 0.0, eps)
    # the library routine keeps the running estimates itself (in place, while training) and
    # normalises with them when training is False
    return F.batch_norm(z, run[name][0], run[name][1], p[name + ".bn.gamma"], p[name + ".bn.beta"], training,
                        momentum, eps)


def forward_blocks(blocks, params, x, labels=None, eps=1e-5, running=None, training=True, momentum=0.1,
                   want_logits=False):
    """Returns the module output, or the mean cross-entropy if the last block is a head (with
    want_logits: (loss, logits)). running: per-block dicts from new_running, updated in place
    when training, used for normalisation when not."""
    logits = None
    for i, (b, p) in enumerate(zip(blocks, params)):
        r = running[i] if running is not None else None
        kw = dict(run=r, training=training, momentum=momentum)
        if b.kind == BLOCK_STEM:
            x = F.relu(_unit(x, p, "conv1", b.stride, eps, **kw))
        elif b.kind == BLOCK_BASIC:
            o = F.relu(_unit(x, p, "conv1", b.stride, eps, **kw))
            z = _unit(o, p, "conv2", 1, eps, **kw)
            sc = _unit(x, p, "proj", b.stride, eps, **kw) if b.projection else x
            x = F.relu(z + sc)
        elif b.kind == BLOCK_BOTTLENECK:
            o = F.relu(_unit(x, p, "conv1", 1, eps, **kw))
            o = F.relu(_unit(o, p, "conv2", b.stride, eps, **kw))
            z = _unit(o, p, "conv3", 1, eps, **kw)
            sc = _unit(x, p, "proj", b.stride, eps, **kw) if b.projection else x
            x = F.relu(z + sc)
        elif b.kind == BLOCK_HEAD:
            pooled = x.mean((2, 3))
            logits = pooled @ p["fc.W"].t() + p["fc.b"]
            x = F.cross_entropy(logits, torch.as_tensor(labels, dtype=torch.long))
    return (x, logits) if want_logits else x
