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


def _unit(x, p, name, stride, eps):
    w = p[name + ".W"]
    pad = 1 if w.shape[-1] == 3 else 0
    z = F.conv2d(x, w, stride=stride, padding=pad)
    return F.batch_norm(z, None, None, p[name + ".bn.gamma"], p[name + ".bn.beta"], True, 0.0, eps)


def forward_blocks(blocks, params, x, labels=None, eps=1e-5):
    """Returns the module output, or the mean cross-entropy if the last block is a head."""
    for b, p in zip(blocks, params):
        if b.kind == BLOCK_STEM:
            x = F.relu(_unit(x, p, "conv1", b.stride, eps))
        elif b.kind == BLOCK_BASIC:
            o = F.relu(_unit(x, p, "conv1", b.stride, eps))
            z = _unit(o, p, "conv2", 1, eps)
            sc = _unit(x, p, "proj", b.stride, eps) if b.projection else x
            x = F.relu(z + sc)
        elif b.kind == BLOCK_BOTTLENECK:
            o = F.relu(_unit(x, p, "conv1", 1, eps))
            o = F.relu(_unit(o, p, "conv2", b.stride, eps))
            z = _unit(o, p, "conv3", 1, eps)
            sc = _unit(x, p, "proj", b.stride, eps) if b.projection else x
            x = F.relu(z + sc)
        elif b.kind == BLOCK_HEAD:
            pooled = x.mean((2, 3))
            logits = pooled @ p["fc.W"].t() + p["fc.b"]
            x = F.cross_entropy(logits, torch.as_tensor(labels, dtype=torch.long))
    return x
