"""Shared test plumbing: build an oracle for a workload, tiny pattern workloads,
error norms.  No arithmetic of the method lives here."""
import numpy as np

from oracle import pbd_oracle as orc
from paper_2301_12443_amd import workloads as W


def make_oracle(wl, batch=None, precision=64):
    words, pool = W.pack(wl)
    o = orc.Oracle(words, pool, wl.batch if batch is None else batch, precision=precision,
                   momentum=wl.momentum)
    for net, b, j, slot, arr in W.iter_params(wl):
        o.set_param(net, b, j, slot, arr)
    return o


def max_rel(a, b):
    """max-norm relative error: max|a-b| / max|b|."""
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    den = np.max(np.abs(b)) if b.size else 0.0
    if den == 0.0:
        return float(np.max(np.abs(a))) if a.size else 0.0
    return float(np.max(np.abs(a - b)) / den)


def pattern_workloads():
    """Tiny instances of every op pattern the five configurations use."""
    out = []
    # depthwise-separable + pool (VGG student), dense 3x3 + pool teacher
    t, s = W.Block(), W.Block()
    v = t.cba(0, 6, 3); v = t.cba(v, 6, 3); t.pool(v, 2, 2)
    v = s.cba(0, 4, 3, groups=4); v = s.cba(v, 6, 1)
    v = s.cba(v, 6, 3, groups=6); v = s.cba(v, 6, 1); s.pool(v, 2, 2)
    out.append(W.Workload("p_dsconv", 3, (4, 8, 8), [t], [s], "f32", lr=0.05))
    # MBConv k3 teacher with residual, MBConv k5/k7 stride 2 + stride-1 residual student
    t, s = W.Block(), W.Block()
    v = W._mbconv(t, 0, 4, 6, 3, 6, 2); W._mbconv(t, v, 6, 6, 3, 6, 1)
    v = W._mbconv(s, 0, 4, 6, 5, 4, 2); W._mbconv(s, v, 6, 6, 7, 3, 1)
    out.append(W.Workload("p_mbconv", 3, (4, 9, 9), [t], [s], "f32", lr=0.05))
    # 7x7 stem + 3x3 s2 p1 pool + bottlenecks with and without projection
    t, s = W.Block(), W.Block()
    for blk, inner in ((t, 4), (s, 6)):
        v = blk.cba(0, 8, 7, 2); v = blk.pool(v, 3, 2, 1)
        v = W._bottleneck(blk, v, 8, inner, 16, 2)
        W._bottleneck(blk, v, 16, inner, 16, 1)
    out.append(W.Workload("p_bottleneck", 2, (3, 20, 20), [t], [s], "f32", lr=0.05))
    # supernet layer: mix of candidates, then a mixed layer with identity skip
    t, s = W.Block(), W.Block()
    v = W._mbconv(t, 0, 4, 6, 3, 6, 2); W._mbconv(t, v, 6, 6, 3, 6, 1)
    cands = ((3, 3), (5, 6), (7, 3))
    p = (0.5, 0.3, 0.2)
    outs = [W._mbconv(s, 0, 4, 6, k, e, 2, residual=False) for k, e in cands]
    v = s.mix(outs, p)
    outs = [W._mbconv(s, v, 6, 6, k, e, 1, residual=False) for k, e in cands]
    m = s.mix(outs, p); s.add(v, m)
    out.append(W.Workload("p_supernet", 2, (4, 8, 8), [t], [s], "f32", lr=0.05))
    return out
