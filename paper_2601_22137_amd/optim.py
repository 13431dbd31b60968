"""Optimizer-side helpers on top of the C-ABI: one grouped library call per optimizer step.

Argument marshalling only: tensors are grouped by shape, stacked into [batch, m, n] arrays (device
copies made by PyTorch) and handed to prism_run_grouped; every step of the method runs in the HIP
kernels.  Nothing here is used by the tests of the hot path or by bench.py's timed region.
"""
import collections

import torch

from . import prism


def _by_shape(tensors):
    groups = collections.OrderedDict()
    for i, t in enumerate(tensors):
        groups.setdefault((tuple(t.shape), t.dtype), []).append(i)
    return groups


def muon_orthogonalize(grads, degree=5, iters=5, sketch_dim=16, seed=22137, warm_iters=0, plain_bf16=True):
    """Polar factors of a list of 2-D gradient / momentum matrices (any mix of shapes, one dtype):
    the orthogonalisation step of a Muon-style optimizer (paper Section 6.2: a fixed small budget
    of PRISM iterations, optionally the first `warm_iters` of them at alpha = u without a fit).
    Returns new tensors in the order of `grads`."""
    prism.lib()
    if len(grads) == 0:
        return []
    groups = _by_shape(grads)
    stacked = [torch.stack([grads[i] for i in idx]).contiguous() for idx in groups.values()]
    flags = prism.FLAG_BF16_PLAIN_ITERATE if (plain_bf16 and stacked[0].dtype == torch.bfloat16) else 0
    prism.run_grouped(prism.FN_POLAR, stacked, degree, iters, sketch_dim, seed, 0.0, flags=flags, warm_iters=warm_iters)
    out = [None] * len(grads)
    for idx, s in zip(groups.values(), stacked):
        for j, i in enumerate(idx):
            out[i] = s[j]
    return out


def shampoo_inverse_roots(stats, root_p=4, max_iters=40, sketch_dim=16, seed=22137, tol=1e-5):
    """A^(-1/root_p) of a list of symmetric positive definite fp32 preconditioner statistics (any mix of
    sizes): the root step of a Shampoo-style optimizer (paper Section 6.2, coupled inverse Newton).
    Returns (roots in the order of `stats`, per-matrix iteration counts)."""
    prism.lib()
    if len(stats) == 0:
        return [], []
    groups = _by_shape(stats)
    stacked = [torch.stack([stats[i] for i in idx]).contiguous() for idx in groups.values()]
    _, infos = prism.run_grouped(prism.FN_INV_ROOT, stacked, 3, max_iters, sketch_dim, seed, tol, root_p=root_p)
    out, iters = [None] * len(stats), [0] * len(stats)
    for idx, s, h in zip(groups.values(), stacked, infos):
        rec = h.read()
        for j, i in enumerate(idx):
            out[i] = s[j]
            iters[i] = int(rec[j]["iters"])
    return out, iters
