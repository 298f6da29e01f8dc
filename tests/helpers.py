"""Shared test plumbing: build an oracle for a workload, tiny pattern workloads,
error norms.  No arithmetic of the method lives here."""
import numpy as np

from oracle import pbd_oracle as orc
from paper_2301_12443_amd import workloads as W


def make_oracle(wl, batch=None, precision=64, storage=None):
    words, pool = W.pack(wl)
    o = orc.Oracle(words, pool, wl.batch if batch is None else batch, precision=precision,
                   momentum=wl.momentum, storage=storage)
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
    """Tiny instances of every op pattern the five configurations use (channel counts are
    multiples of 8 past the input, as the device layout wants)."""
    out = []
    # depthwise-separable + pool (VGG student) on a 3-channel input, dense 3x3 + pool teacher
    t, s = W.Block(), W.Block()
    v = t.cba(0, 8, 3); v = t.cba(v, 8, 3); t.pool(v, 2, 2)
    v = s.cba(0, 3, 3, groups=3); v = s.cba(v, 8, 1)
    v = s.cba(v, 8, 3, groups=8); v = s.cba(v, 8, 1); s.pool(v, 2, 2)
    out.append(W.Workload("p_dsconv", 3, (3, 8, 8), [t], [s], "f32", lr=0.05))
    # MBConv k3 teacher with residual, MBConv k5/k7 stride 2 + stride-1 residual student
    t, s = W.Block(), W.Block()
    v = W._mbconv(t, 0, 8, 16, 3, 6, 2); W._mbconv(t, v, 16, 16, 3, 6, 1)
    v = W._mbconv(s, 0, 8, 16, 5, 4, 2); W._mbconv(s, v, 16, 16, 7, 3, 1)
    out.append(W.Workload("p_mbconv", 3, (8, 9, 9), [t], [s], "f32", lr=0.05))
    # 7x7 stem + 3x3 s2 p1 pool + bottlenecks with and without projection
    t, s = W.Block(), W.Block()
    for blk, inner in ((t, 8), (s, 16)):
        v = blk.cba(0, 8, 7, 2); v = blk.pool(v, 3, 2, 1)
        v = W._bottleneck(blk, v, 8, inner, 16, 2)
        W._bottleneck(blk, v, 16, inner, 16, 1)
    out.append(W.Workload("p_bottleneck", 2, (3, 20, 20), [t], [s], "f32", lr=0.05))
    # supernet layer: mix of candidates, then a mixed layer with identity skip
    t, s = W.Block(), W.Block()
    v = W._mbconv(t, 0, 8, 16, 3, 6, 2); W._mbconv(t, v, 16, 16, 3, 6, 1)
    cands = ((3, 3), (5, 6), (7, 3))
    p = (0.5, 0.3, 0.2)
    outs = [W._mbconv(s, 0, 8, 16, k, e, 2, residual=False) for k, e in cands]
    v = s.mix(outs, p)
    outs = [W._mbconv(s, v, 16, 16, k, e, 1, residual=False) for k, e in cands]
    m = s.mix(outs, p); s.add(v, m)
    out.append(W.Workload("p_supernet", 2, (8, 8, 8), [t], [s], "f32", lr=0.05))
    return out


def layer_workloads():
    """Two-to-four-op student blocks at the layer shapes of the five configurations
    (channel counts, kernel sizes, strides, ragged row and column counts), shallow enough that
    bf16 storage noise is not amplified by depth.  Returned as (workload, batch) pairs."""
    out = []

    def wl(name, in_shape, t, s, batch):
        out.append((W.Workload(name, batch, in_shape, [t], [s], "bf16", lr=0.05), batch))

    # dense 3x3, K = 576, 128 full row tiles (VGG teacher shape as a student layer)
    t, s = W.Block(), W.Block()
    t.cba(0, 64, 3)
    v = s.cba(0, 64, 1); s.cba(v, 64, 3)
    wl("l_dense3x3", (64, 16, 16), t, s, 64)
    # ragged rows (980) and columns (40, 72), stride-2 3x3 with backward-data
    t, s = W.Block(), W.Block()
    t.cba(0, 72, 3, 2)
    v = s.cba(0, 40, 1); s.cba(v, 72, 3, 2)
    wl("l_ragged_s2", (24, 14, 14), t, s, 5)
    # depthwise-separable chain with pooling (VGG student)
    t, s = W.Block(), W.Block()
    v = t.cba(0, 128, 3); t.pool(v, 2, 2)
    v = s.cba(0, 64, 3, groups=64); v = s.cba(v, 128, 1)
    v = s.cba(v, 128, 3, groups=128); v = s.cba(v, 128, 1); s.pool(v, 2, 2)
    wl("l_dsconv", (64, 16, 16), t, s, 64)
    # 3-channel input: 7x7 stride-2 stem, 3x3 s2 p1 pool, 1x1 (ResNet stem; even image size: the library runs it as a
    # 4 x 4 stride-1 convolution over a space-to-depth copy of the input)
    t, s = W.Block(), W.Block()
    v = t.cba(0, 64, 7, 2); t.pool(v, 3, 2, 1)
    v = s.cba(0, 64, 7, 2); v = s.pool(v, 3, 2, 1); s.cba(v, 64, 1)
    wl("l_stem7x7", (3, 64, 64), t, s, 8)
    # the same stem on an odd image size: no space-to-depth copy of the input, the 7 x 7 filter is run as it is
    t, s = W.Block(), W.Block()
    v = t.cba(0, 64, 7, 2); t.pool(v, 3, 2, 1)
    v = s.cba(0, 64, 7, 2); v = s.pool(v, 3, 2, 1); s.cba(v, 64, 1)
    wl("l_stem7x7_odd", (3, 45, 45), t, s, 8)
    # MBConv k5 stride 2 (MobileNet student) and k7 stride 1 with residual (supernet candidate)
    t, s = W.Block(), W.Block()
    W._mbconv(t, 0, 24, 32, 3, 6, 2)
    W._mbconv(s, 0, 24, 32, 5, 4, 2)
    wl("l_mbconv_k5s2", (24, 28, 28), t, s, 16)
    t, s = W.Block(), W.Block()
    W._mbconv(t, 0, 32, 32, 3, 6, 1)
    W._mbconv(s, 0, 32, 32, 7, 3, 1)
    wl("l_mbconv_k7res", (32, 14, 14), t, s, 16)
    # wide 1x1 layers, small row count (ResNet stage 4 shape)
    t, s = W.Block(), W.Block()
    t.cba(0, 1024, 1)
    v = s.cba(0, 384, 1); s.cba(v, 1024, 1, act=W.ACT_NONE)
    wl("l_wide1x1", (512, 7, 7), t, s, 32)
    # deep reduction: 3x3 over 384 channels (K = 3456) with backward-data
    t, s = W.Block(), W.Block()
    t.cba(0, 384, 3)
    v = s.cba(0, 384, 1); s.cba(v, 384, 3)
    wl("l_deepK3x3", (256, 7, 7), t, s, 32)
    # long columns: 147456 rows = 1152 row tiles, more partial sums than one normalisation finalize walks
    t, s = W.Block(), W.Block()
    t.cba(0, 16, 3)
    v = s.cba(0, 40, 1); s.cba(v, 16, 3)
    wl("l_long_column", (24, 64, 64), t, s, 36)
    # a long column that is no multiple of any tile height: 18000 rows (70 tiles of 256 rows and a ragged 80-row one)
    t, s = W.Block(), W.Block()
    t.cba(0, 64, 3)
    v = s.cba(0, 40, 1); s.cba(v, 64, 3)
    wl("l_ragged_long", (24, 60, 60), t, s, 5)
    # stride-2 3 x 3 and stride-2 1 x 1 that both read an interior value (a bottleneck with projection shortcut
    # in the middle of a block): their backward-data launches take the input pixels parity class by parity class,
    # one storing (for the 1 x 1: three classes of zeros), one adding onto it; 25392 rows a class (99 tiles and a
    # ragged one), in both orders
    for name, shortcut_first in (("l_s2_classes", False), ("l_s2_classes_swapped", True)):
        t, s = W.Block(), W.Block()
        t.cba(0, 256, 3, 2)
        v1 = s.cba(0, 192, 1)
        if shortcut_first:
            sc = s.cba(v1, 256, 1, 2, act=W.ACT_NONE)
        v = s.cba(v1, 64, 3, 2); v = s.cba(v, 256, 1, act=W.ACT_NONE)
        if not shortcut_first:
            sc = s.cba(v1, 256, 1, 2, act=W.ACT_NONE)
        s.add(v, sc, W.ACT_RELU)
        wl(name, (24, 46, 46), t, s, 48)
    # an inverted-residual block whose skip is the block's input (no gradient wanted there) and whose add is the
    # block's last op: 6272 pixels, so the add's backward pass and the loss ride in the projection's batch-norm
    # backward reduction
    t, s = W.Block(), W.Block()
    W._mbconv(t, 0, 32, 32, 3, 6, 1)
    W._mbconv(s, 0, 32, 32, 7, 3, 1)
    wl("l_res_from_input", (32, 14, 14), t, s, 32)
    # two fused adds, 6400 pixels: the last one carries the loss; the first one's skip input already holds a
    # gradient when its turn comes (a later layer reads the same value), so it keeps the separate add backward
    t, s = W.Block(), W.Block()
    t.cba(0, 24, 3)
    v1 = s.cba(0, 24, 1)
    c = s.cba(v1, 24, 3, act=W.ACT_NONE)
    a = s.add(v1, c, W.ACT_RELU)
    e = s.cba(v1, 24, 1, act=W.ACT_NONE)
    s.add(a, e, W.ACT_RELU)
    wl("l_add_bwd_paths", (24, 20, 20), t, s, 16)
    return out


def supernet():
    """The tiny two-layer supernet block of pattern_workloads()."""
    return next(w for w in pattern_workloads() if w.name == "p_supernet")


def mix_ops(wl, b=0):
    return [(j, len(op.inputs)) for j, op in enumerate(wl.student[b].ops) if op.type == W.OP_MIX]


def twin_candidates(n=3, act=W.ACT_NONE):
    """A mix of n candidates of one shape (dense 3x3 -> 1x1), then a rectified residual sum."""
    t, s = W.Block(), W.Block()
    t.cba(0, 8, 3)
    outs = []
    for _ in range(n):
        v = s.cba(0, 16, 3)
        outs.append(s.cba(v, 8, 1, act=W.ACT_NONE))
    m = s.mix(outs, [1.0 / n] * n)
    v = s.cba(m, 8, 3)
    s.add(m, v, act=act)
    return W.Workload("twins", 3, (8, 6, 6), [t], [s], "f32", lr=0.05)


def skip_mix():
    """A mix whose first candidate is the block's input itself, then a mix over a single candidate."""
    t, s = W.Block(), W.Block()
    t.cba(0, 8, 3)
    a = s.cba(0, 8, 3, act=W.ACT_NONE)
    v = s.cba(0, 16, 1); b = s.cba(v, 8, 3, act=W.ACT_NONE)
    m = s.mix([0, a, b], [0.2, 0.5, 0.3])
    c = s.cba(m, 8, 3)
    s.mix([c], [1.0])
    return W.Workload("skip_mix", 4, (8, 6, 6), [t], [s], "f32", lr=0.05)
