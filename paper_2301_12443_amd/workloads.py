"""Workload descriptors and seeded synthetic inputs for blockwise distillation.

This module is pure data: it lists, for each benchmark configuration, the
teacher blocks T_i and student blocks S_i (Sec. II-A: every (T_i, S_i) pair maps
the previous teacher activation A_{i-1} to tensors of one common shape), packs
them into a flat int32/float64 wire format, and draws the synthetic inputs and
parameters from a seed.  It holds none of the method's arithmetic (no
convolution, normalisation, loss or optimiser code); the CPU oracle and the HIP
library each parse the wire format on their own.

Operation vocabulary (value 0 of a block is its input A_{i-1}; op j produces
value j+1; the block output is the last value):

  CBA   convolution (square kernel k, stride s, zero pad k//2, groups 1 or C_in,
        no bias) followed by batch normalisation and an activation
        (0 none, 1 ReLU, 2 ReLU6)
  POOL  max pooling (k, stride, pad)
  ADD   elementwise sum of two values followed by an activation
  MIX   weighted sum  y = sum_k p_k * v_k  of several values (NAS supernet layer,
        Sec. VI-A: every candidate operation carries a selection probability)
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

import numpy as np

MAGIC = 0x50424431  # "PBD1"
REC = 20            # int32 words per op record
OP_CBA, OP_POOL, OP_ADD, OP_MIX = 1, 2, 3, 4
ACT_NONE, ACT_RELU, ACT_RELU6 = 0, 1, 2
NET_TEACHER, NET_STUDENT = 0, 1
# parameter slots of a CBA op
P_WEIGHT, P_GAMMA, P_BETA, P_RMEAN, P_RVAR = 0, 1, 2, 3, 4


@dataclass
class Op:
    type: int
    inputs: Tuple[int, ...]
    c_out: int = 0
    k: int = 0
    stride: int = 1
    pad: int = 0
    groups: int = 1
    act: int = ACT_NONE
    p: Tuple[float, ...] = ()


@dataclass
class Block:
    ops: List[Op] = field(default_factory=list)

    # tiny builder helpers: each returns the id of the value it produced
    def cba(self, x: int, c_out: int, k: int, stride: int = 1, groups: int = 1,
            act: int = ACT_RELU) -> int:
        self.ops.append(Op(OP_CBA, (x,), c_out=c_out, k=k, stride=stride,
                           pad=k // 2, groups=groups, act=act))
        return len(self.ops)

    def pool(self, x: int, k: int, stride: int, pad: int = 0) -> int:
        self.ops.append(Op(OP_POOL, (x,), k=k, stride=stride, pad=pad))
        return len(self.ops)

    def add(self, a: int, b: int, act: int = ACT_NONE) -> int:
        self.ops.append(Op(OP_ADD, (a, b), act=act))
        return len(self.ops)

    def mix(self, xs: Sequence[int], p: Sequence[float]) -> int:
        assert len(xs) == len(p) and 1 <= len(xs) <= 8
        self.ops.append(Op(OP_MIX, tuple(xs), p=tuple(float(v) for v in p)))
        return len(self.ops)


@dataclass
class Workload:
    name: str
    batch: int
    in_shape: Tuple[int, int, int]          # C, H, W of A_0
    teacher: List[Block]
    student: List[Block]
    precision: str                          # "f32" or "bf16"
    lr: float
    momentum: float = 0.9
    seed: int = 2301

    @property
    def B(self) -> int:
        return len(self.teacher)

    def net(self, which: int) -> List[Block]:
        return self.teacher if which == NET_TEACHER else self.student


# ----------------------------------------------------------------------------
# shape walking (integer bookkeeping only)
# ----------------------------------------------------------------------------

def out_hw(h: int, k: int, stride: int, pad: int) -> int:
    return (h + 2 * pad - k) // stride + 1


def block_shapes(block: Block, in_shape: Tuple[int, int, int]) -> List[Tuple[int, int, int]]:
    """(C, H, W) of every value of a block, value 0 first."""
    shapes = [tuple(in_shape)]
    for op in block.ops:
        c, h, w = shapes[op.inputs[0]]
        if op.type == OP_CBA:
            assert op.groups in (1, c), "groups must be 1 or C_in"
            if op.groups != 1:
                assert op.c_out == c, "depthwise keeps the channel count"
            shapes.append((op.c_out, out_hw(h, op.k, op.stride, op.pad),
                           out_hw(w, op.k, op.stride, op.pad)))
        elif op.type == OP_POOL:
            shapes.append((c, out_hw(h, op.k, op.stride, op.pad),
                           out_hw(w, op.k, op.stride, op.pad)))
        elif op.type in (OP_ADD, OP_MIX):
            for j in op.inputs:
                assert shapes[j] == (c, h, w), "joined values must agree in shape"
            shapes.append((c, h, w))
        else:
            raise ValueError(op.type)
    return shapes


def activation_shapes(wl: Workload) -> List[Tuple[int, int, int]]:
    """Shapes of A_0..A_B; also checks that T_i and S_i agree (Sec. II-A)."""
    shapes = [tuple(wl.in_shape)]
    for tb, sb in zip(wl.teacher, wl.student):
        t_out = block_shapes(tb, shapes[-1])[-1]
        s_out = block_shapes(sb, shapes[-1])[-1]
        assert t_out == s_out, (wl.name, t_out, s_out)
        shapes.append(t_out)
    return shapes


def param_shapes(wl: Workload, net: int, b: int) -> Dict[Tuple[int, int], Tuple[int, ...]]:
    """{(op index, slot): shape} of every parameter tensor of block b (0-based)."""
    a_shapes = activation_shapes(wl)
    block = wl.net(net)[b]
    shapes = block_shapes(block, a_shapes[b])
    out = {}
    for j, op in enumerate(block.ops):
        if op.type != OP_CBA:
            continue
        c_in = shapes[op.inputs[0]][0]
        out[(j, P_WEIGHT)] = (op.c_out, c_in // op.groups, op.k, op.k)
        for slot in (P_GAMMA, P_BETA, P_RMEAN, P_RVAR):
            out[(j, slot)] = (op.c_out,)
    return out


def macs_and_params(blocks: List[Block], in_shape, trainable_only=True):
    """Per-block (dense MACs, depthwise MACs, parameter count) per sample."""
    res = []
    shp = tuple(in_shape)
    for block in blocks:
        shapes = block_shapes(block, shp)
        dense = dw = params = 0
        for j, op in enumerate(block.ops):
            if op.type != OP_CBA:
                continue
            c_in = shapes[op.inputs[0]][0]
            c, h, w = shapes[j + 1]
            m = (c_in // op.groups) * op.k * op.k * c * h * w
            if op.groups == 1:
                dense += m
            else:
                dw += m
            params += op.c_out * (c_in // op.groups) * op.k * op.k + 2 * op.c_out
        res.append((dense, dw, params))
        shp = shapes[-1]
    return res


# ----------------------------------------------------------------------------
# wire format
# ----------------------------------------------------------------------------

def pack(wl: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """Flat (int32 words, float64 pool) description of both networks.

    words: MAGIC, version, B, C0, H0, W0, then for the teacher and then the
    student, for every block: n_ops followed by n_ops records of REC words:
    [type, n_in, in0..in7, c_out, k, stride, pad, groups, act, p_offset, 0, 0, 0]
    where p_offset indexes the float pool (MIX weights).
    """
    activation_shapes(wl)  # validates
    words: List[int] = [MAGIC, 1, wl.B, *wl.in_shape]
    pool: List[float] = []
    for blocks in (wl.teacher, wl.student):
        for block in blocks:
            words.append(len(block.ops))
            for op in block.ops:
                ins = list(op.inputs) + [0] * (8 - len(op.inputs))
                rec = [op.type, len(op.inputs), *ins, op.c_out, op.k, op.stride,
                       op.pad, op.groups, op.act, len(pool), 0, 0, 0]
                assert len(rec) == REC
                words.extend(rec)
                pool.extend(op.p)
    return np.asarray(words, dtype=np.int32), np.asarray(pool + [0.0], dtype=np.float64)


# ----------------------------------------------------------------------------
# seeded synthetic data
# ----------------------------------------------------------------------------

def _rng(wl: Workload, *key: int) -> np.random.Generator:
    return np.random.default_rng([wl.seed, *[int(k) for k in key]])


def make_input(wl: Workload, batch: int | None = None, step: int = 0) -> np.ndarray:
    """x ~ N(0,1), float32, NCHW; stands in for CIFAR-10 / ImageNet images."""
    n = wl.batch if batch is None else batch
    return _rng(wl, 7, step).standard_normal((n, *wl.in_shape), dtype=np.float32)


def _is_linear_value(wl: Workload, net: int, b: int, v: int) -> bool:
    """True when value v of block b comes out of a layer without a rectifier."""
    if v == 0:
        if b == 0:
            return False                      # the image: plain He-normal first layer
        last = wl.teacher[b - 1].ops[-1]      # A_{i-1} is the teacher's output for both nets
        return last.type in (OP_ADD, OP_CBA) and last.act == ACT_NONE or last.type == OP_MIX
    op = wl.net(net)[b].ops[v - 1]
    if op.type == OP_POOL:
        return _is_linear_value(wl, net, b, op.inputs[0])
    return op.type == OP_MIX or op.act == ACT_NONE


def _feeds_add(block: Block, j: int) -> bool:
    return any(o.type == OP_ADD and (j + 1) in o.inputs for o in block.ops)


def make_param(wl: Workload, net: int, b: int, j: int, slot: int,
               shape: Tuple[int, ...]) -> np.ndarray:
    """One parameter tensor (float32), regenerable on its own from the seed.

    Conv weights: He-normal, std = sqrt(gain / fan_in) with gain 2 behind a rectifier and
    gain 1 behind a linear output (linear bottleneck, residual sum, mix), which keeps
    activations at unit scale through deep inverted-residual stacks the way a trained
    network's statistics do.  Student BN starts at the identity (gamma 1, beta 0, running
    mean 0, running var 1).  The frozen teacher BN gets non-trivial values so that a wrong
    fold cannot hide: gamma ~ U(0.5,1.5) (halved on the last BN of a residual branch, as
    trained residual networks have small branch gains), beta ~ N(0,0.1^2),
    mean ~ N(0,0.1^2), var ~ U(0.5,1.5).
    """
    g = _rng(wl, net, b, j, slot)
    block = wl.net(net)[b]
    if slot == P_WEIGHT:
        fan_in = shape[1] * shape[2] * shape[3]
        gain = 1.0 if _is_linear_value(wl, net, b, block.ops[j].inputs[0]) else 2.0
        w = g.standard_normal(shape, dtype=np.float32)
        return (w * np.float32(np.sqrt(gain / fan_in))).astype(np.float32)
    if net == NET_STUDENT:
        fill = {P_GAMMA: 1.0, P_BETA: 0.0, P_RMEAN: 0.0, P_RVAR: 1.0}[slot]
        return np.full(shape, fill, dtype=np.float32)
    if slot == P_GAMMA:
        scale = 0.5 if (block.ops[j].act == ACT_NONE and _feeds_add(block, j)) else 1.0
        return (scale * g.uniform(0.5, 1.5, shape)).astype(np.float32)
    if slot == P_RVAR:
        return g.uniform(0.5, 1.5, shape).astype(np.float32)
    return (0.1 * g.standard_normal(shape)).astype(np.float32)


def iter_params(wl: Workload):
    """Yield (net, block, op, slot, array) for every parameter of both nets."""
    for net in (NET_TEACHER, NET_STUDENT):
        for b in range(wl.B):
            for (j, slot), shape in param_shapes(wl, net, b).items():
                yield net, b, j, slot, make_param(wl, net, b, j, slot, shape)


# ----------------------------------------------------------------------------
# the five configurations
# ----------------------------------------------------------------------------

def tiny_cnn(batch: int = 8) -> Workload:
    widths, strides = (16, 32, 64, 128), (1, 2, 2, 2)
    teacher, student = [], []
    for w, s in zip(widths, strides):
        t = Block(); t.cba(0, w, 3, s)
        st = Block(); v = st.cba(0, w // 2, 3, s); st.cba(v, w, 1)
        teacher.append(t); student.append(st)
    return Workload("tiny_cnn", batch, (3, 32, 32), teacher, student, "f32", lr=0.01)


_VGG_BLOCKS = ((64, 64, "M"), (128, 128, "M"), (256, 256, 256, "M"),
               (512, 512, 512, "M", 512, 512, 512, "M"))


def vgg16_dsconv(batch: int = 256, hw: int = 32, precision: str = "bf16") -> Workload:
    teacher, student = [], []
    c_in = 3
    for stage in _VGG_BLOCKS:
        t, s = Block(), Block()
        tv = sv = 0
        for item in stage:
            if item == "M":
                tv = t.pool(tv, 2, 2)
                sv = s.pool(sv, 2, 2)
            else:
                tv = t.cba(tv, item, 3)
                sv = s.cba(sv, c_in, 3, groups=c_in)     # depthwise 3x3
                sv = s.cba(sv, item, 1)                  # pointwise 1x1
                c_in = item
        teacher.append(t); student.append(s)
    return Workload("vgg16_dsconv", batch, (3, hw, hw), teacher, student, precision, lr=0.1)


def _mbconv(b: Block, x: int, c_in: int, c_out: int, k: int, e: float, stride: int,
            residual: bool = True) -> int:
    v = x
    if e != 1:
        v = b.cba(v, int(round(e * c_in)), 1, act=ACT_RELU6)
    mid = int(round(e * c_in))
    v = b.cba(v, mid, k, stride, groups=mid, act=ACT_RELU6)
    v = b.cba(v, c_out, 1, act=ACT_NONE)
    if residual and stride == 1 and c_in == c_out:
        v = b.add(x, v)
    return v


# MobileNetV2-1.0 body, grouped into six blocks: (expansion, channels, repeats, stride)
_MBV2_BLOCKS = (((1, 16, 1, 1),), ((6, 24, 2, 2),), ((6, 32, 3, 2),), ((6, 64, 4, 2),),
                ((6, 96, 3, 1),), ((6, 160, 3, 2), (6, 320, 1, 1)))


def _mbv2_teacher() -> List[Block]:
    blocks = []
    c_in = 32
    for bi, groups in enumerate(_MBV2_BLOCKS):
        b = Block()
        v = 0
        if bi == 0:
            v = b.cba(0, 32, 3, 2, act=ACT_RELU6)
        for (t, c, n, s) in groups:
            for r in range(n):
                v = _mbconv(b, v, c_in, c, 3, t, s if r == 0 else 1)
                c_in = c
        blocks.append(b)
    return blocks


def mbv2_mbconv(batch: int = 128, hw: int = 224, precision: str = "bf16") -> Workload:
    student = []
    c_in = 32
    for bi, groups in enumerate(_MBV2_BLOCKS):
        b = Block()
        v = 0
        if bi == 0:
            v = b.cba(0, 32, 3, 2, act=ACT_RELU6)
        for (_, c, n, s) in groups:
            for r in range(n):
                v = _mbconv(b, v, c_in, c, 5, 4, s if r == 0 else 1)
                c_in = c
        student.append(b)
    return Workload("mbv2_mbconv_k5e4", batch, (3, hw, hw), _mbv2_teacher(), student,
                    precision, lr=0.005)


_NAS_CANDIDATES = tuple((k, e) for k in (3, 5, 7) for e in (3, 6))


def mbv2_supernet(batch: int = 64, hw: int = 224, precision: str = "bf16") -> Workload:
    student = []
    c_in = 32
    p = [1.0 / len(_NAS_CANDIDATES)] * len(_NAS_CANDIDATES)   # softmax of alpha = 0
    for bi, groups in enumerate(_MBV2_BLOCKS):
        b = Block()
        v = 0
        if bi == 0:
            v = b.cba(0, 32, 3, 2, act=ACT_RELU6)
        c_out = groups[-1][1]
        stride = groups[0][3]
        for layer in range(4):
            s = stride if layer == 0 else 1
            outs = [_mbconv(b, v, c_in, c_out, k, e, s, residual=False)
                    for (k, e) in _NAS_CANDIDATES]
            m = b.mix(outs, p)
            v = b.add(v, m) if layer > 0 else m
            c_in = c_out
        student.append(b)
    return Workload("mbv2_supernet", batch, (3, hw, hw), _mbv2_teacher(), student,
                    precision, lr=0.005)


def _bottleneck(b: Block, x: int, c_in: int, inner: int, c_out: int, stride: int) -> int:
    v = b.cba(x, inner, 1)
    v = b.cba(v, inner, 3, stride)
    v = b.cba(v, c_out, 1, act=ACT_NONE)
    sc = x
    if stride != 1 or c_in != c_out:
        sc = b.cba(x, c_out, 1, stride, act=ACT_NONE)
    return b.add(sc, v, act=ACT_RELU)


def _resnet50(inner_scale: float) -> List[Block]:
    blocks = []
    c_in = 64
    for si, (w, n, s) in enumerate(((64, 3, 1), (128, 4, 2), (256, 6, 2), (512, 3, 2))):
        b = Block()
        v = 0
        if si == 0:
            v = b.cba(0, 64, 7, 2)
            v = b.pool(v, 3, 2, 1)
        for r in range(n):
            v = _bottleneck(b, v, c_in, int(round(w * inner_scale)), 4 * w, s if r == 0 else 1)
            c_in = 4 * w
        blocks.append(b)
    return blocks


def resnet50_wide(batch: int = 256, hw: int = 224, precision: str = "bf16") -> Workload:
    return Workload("resnet50_x1.5", batch, (3, hw, hw), _resnet50(1.0), _resnet50(1.5),
                    precision, lr=0.1)


CONFIGS = {
    "tiny_cnn": tiny_cnn,
    "vgg16_dsconv": vgg16_dsconv,
    "mbv2_mbconv_k5e4": mbv2_mbconv,
    "mbv2_supernet": mbv2_supernet,
    "resnet50_x1.5": resnet50_wide,
}
