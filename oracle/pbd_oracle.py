"""ctypes wrapper over the CPU oracle (oracle/pbd_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg; never by the product package.  It takes the packed
descriptor words as plain arrays and imports nothing from the HIP side.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pbd_oracle.cpp")
_LIB = os.path.join(_HERE, "libpbd_oracle.so")

KIND_PARAM, KIND_GRAD, KIND_MOMENTUM = 0, 1, 2
MODE_LOSS, MODE_GRADS, MODE_STEP, MODE_ARCH_GRADS, MODE_ARCH_STEP = 0, 1, 2, 3, 4
ALPHA_VALUE, ALPHA_GRAD, ALPHA_MOMENTUM, ALPHA_PROB = 0, 1, 2, 3

_dp = C.POINTER(C.c_double)
_ip = C.POINTER(C.c_int32)


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (OpenMP) next to its source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-fopenmp", "-shared", "-fPIC",
                               _SRC, "-o", _LIB])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.orc_create.restype = C.c_void_p
        L.orc_create.argtypes = [_ip, C.c_int, _dp, C.c_int, C.c_int, C.c_int,
                                 C.c_double, C.c_double, C.c_double, C.c_int]
        L.orc_destroy.argtypes = [C.c_void_p]
        for f in (L.orc_set_tensor, L.orc_get_tensor):
            f.restype = C.c_int
            f.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _dp, C.c_long]
        L.orc_teacher_relay.argtypes = [C.c_void_p, _dp]
        L.orc_teacher_upto.argtypes = [C.c_void_p, _dp, C.c_int, _dp]
        L.orc_act_numel.restype = C.c_long
        L.orc_act_numel.argtypes = [C.c_void_p, C.c_int]
        L.orc_get_act.argtypes = [C.c_void_p, C.c_int, _dp]
        L.orc_student_step.restype = C.c_double
        L.orc_student_step.argtypes = [C.c_void_p, C.c_int, _dp, _dp, C.c_double, C.c_int]
        L.orc_relay_step.argtypes = [C.c_void_p, _dp, C.c_double, _dp]
        L.orc_redundant_step.argtypes = [C.c_void_p, _dp, C.c_double, _dp]
        L.orc_relay_arch_step.argtypes = [C.c_void_p, _dp, C.c_double, _dp]
        L.orc_set_alpha.restype = C.c_int
        L.orc_set_alpha.argtypes = [C.c_void_p, C.c_int, C.c_int, _dp, C.c_int]
        L.orc_get_alpha.restype = C.c_int
        L.orc_get_alpha.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, _dp, C.c_int]
        L.orc_value_numel.restype = C.c_long
        L.orc_value_numel.argtypes = [C.c_void_p, C.c_int, C.c_int]
        L.orc_get_value.argtypes = [C.c_void_p, C.c_int, C.c_int, _dp]
        L.orc_saved_numel.restype = C.c_long
        L.orc_saved_numel.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int]
        L.orc_get_saved.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, _dp]
        L.orc_round_bf16.argtypes = [_dp, _dp, C.c_long]
        L.orc_kink_margin.restype = C.c_double
        L.orc_kink_margin.argtypes = [C.c_void_p, C.c_int]
        L.orc_num_threads.restype = C.c_int
        conv = [_dp, _dp, _dp] + [C.c_int] * 9
        L.orc_conv_fwd.argtypes = conv
        L.orc_conv_dgrad.argtypes = conv
        L.orc_conv_wgrad.argtypes = conv
        L.orc_bn_train_fwd.argtypes = [_dp] * 6 + [C.c_int] * 3 + [C.c_double]
        L.orc_bn_train_bwd.argtypes = [_dp] * 8 + [C.c_int] * 3 + [C.c_double]
        L.orc_bn_eval.argtypes = [_dp] * 6 + [C.c_int] * 3 + [C.c_double]
        L.orc_act_fwd.argtypes = [_dp, _dp, C.c_long, C.c_int]
        L.orc_act_bwd.argtypes = [_dp, _dp, _dp, C.c_long, C.c_int]
        L.orc_maxpool_fwd.argtypes = [_dp, _dp, _ip] + [C.c_int] * 7
        L.orc_maxpool_bwd.argtypes = [_dp, _ip, _dp] + [C.c_int] * 6
        L.orc_mix_alpha_grad.argtypes = [_dp, _dp, _dp, C.c_int, C.c_long, _dp]
        L.orc_mse.restype = C.c_double
        L.orc_mse.argtypes = [_dp, _dp, _dp, C.c_long]
        L.orc_sgd.argtypes = [_dp, _dp, _dp, C.c_long, C.c_double, C.c_double]
        _lib = L
    return _lib


def _d(a):
    return a.ctypes.data_as(_dp)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def num_threads() -> int:
    return lib().orc_num_threads()


def round_bf16(a):
    """The bf16 mode's storage rounding (nearest even, through float32), elementwise."""
    a = _f64(a)
    out = np.empty_like(a)
    lib().orc_round_bf16(_d(a), _d(out), a.size)
    return out


# --------------------------------------------------------------------------
# primitives (fp64, NCHW)
# --------------------------------------------------------------------------

def _out(h, k, s, p):
    return (h + 2 * p - k) // s + 1


def conv_fwd(x, w, stride=1, pad=0, groups=1):
    x, w = _f64(x), _f64(w)
    N, Cc, H, W = x.shape
    K, _, k, _ = w.shape
    y = np.empty((N, K, _out(H, k, stride, pad), _out(W, k, stride, pad)))
    lib().orc_conv_fwd(_d(x), _d(w), _d(y), N, Cc, H, W, K, k, stride, pad, groups)
    return y


def conv_dgrad(dy, w, x_shape, stride=1, pad=0, groups=1):
    dy, w = _f64(dy), _f64(w)
    N, Cc, H, W = x_shape
    K, _, k, _ = w.shape
    dx = np.empty(x_shape)
    lib().orc_conv_dgrad(_d(dy), _d(w), _d(dx), N, Cc, H, W, K, k, stride, pad, groups)
    return dx


def conv_wgrad(dy, x, k, stride=1, pad=0, groups=1):
    dy, x = _f64(dy), _f64(x)
    N, Cc, H, W = x.shape
    K = dy.shape[1]
    dw = np.empty((K, Cc // groups, k, k))
    lib().orc_conv_wgrad(_d(dy), _d(x), _d(dw), N, Cc, H, W, K, k, stride, pad, groups)
    return dw


def bn_train_fwd(x, gamma, beta, eps=1e-5):
    x, gamma, beta = _f64(x), _f64(gamma), _f64(beta)
    N, Cc = x.shape[:2]
    HW = int(np.prod(x.shape[2:]))
    y = np.empty_like(x)
    mean, var = np.empty(Cc), np.empty(Cc)
    lib().orc_bn_train_fwd(_d(x), _d(gamma), _d(beta), _d(y), _d(mean), _d(var), N, Cc, HW, eps)
    return y, mean, var


def bn_train_bwd(dy, x, gamma, mean, var, eps=1e-5):
    dy, x, gamma, mean, var = map(_f64, (dy, x, gamma, mean, var))
    N, Cc = x.shape[:2]
    HW = int(np.prod(x.shape[2:]))
    dx = np.empty_like(x)
    dg, db = np.empty(Cc), np.empty(Cc)
    lib().orc_bn_train_bwd(_d(dy), _d(x), _d(gamma), _d(mean), _d(var), _d(dx), _d(dg), _d(db),
                           N, Cc, HW, eps)
    return dx, dg, db


def bn_eval(x, gamma, beta, rmean, rvar, eps=1e-5):
    x, gamma, beta, rmean, rvar = map(_f64, (x, gamma, beta, rmean, rvar))
    N, Cc = x.shape[:2]
    HW = int(np.prod(x.shape[2:]))
    y = np.empty_like(x)
    lib().orc_bn_eval(_d(x), _d(gamma), _d(beta), _d(rmean), _d(rvar), _d(y), N, Cc, HW, eps)
    return y


def act_fwd(x, act):
    x = _f64(x)
    y = np.empty_like(x)
    lib().orc_act_fwd(_d(x), _d(y), x.size, act)
    return y


def act_bwd(dy, x, act):
    dy, x = _f64(dy), _f64(x)
    dx = np.empty_like(x)
    lib().orc_act_bwd(_d(dy), _d(x), _d(dx), x.size, act)
    return dx


def maxpool_fwd(x, k, stride, pad=0):
    x = _f64(x)
    N, Cc, H, W = x.shape
    P, Q = _out(H, k, stride, pad), _out(W, k, stride, pad)
    y = np.empty((N, Cc, P, Q))
    idx = np.empty((N, Cc, P, Q), dtype=np.int32)
    lib().orc_maxpool_fwd(_d(x), _d(y), idx.ctypes.data_as(_ip), N, Cc, H, W, k, stride, pad)
    return y, idx


def maxpool_bwd(dy, idx, x_shape):
    dy = _f64(dy)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    N, Cc, H, W = x_shape
    dx = np.empty(x_shape)
    lib().orc_maxpool_bwd(_d(dy), idx.ctypes.data_as(_ip), _d(dx), N, Cc, H, W,
                          dy.shape[2], dy.shape[3])
    return dx


def mix_alpha_grad(dz, ys, p):
    """dL/dalpha of one weighted sum z = sum_k softmax(alpha)_k y_k, from dL/dz, the candidates y_k and p."""
    dz = _f64(dz).ravel()
    ys = np.ascontiguousarray(np.stack([_f64(y).ravel() for y in ys]))
    p = _f64(p).ravel()
    out = np.empty(p.size)
    lib().orc_mix_alpha_grad(_d(dz), _d(ys), _d(p), p.size, dz.size, _d(out))
    return out


def mse(s, t):
    s, t = _f64(s), _f64(t)
    ds = np.empty_like(s)
    loss = lib().orc_mse(_d(s), _d(t), _d(ds), s.size)
    return loss, ds


def sgd(w, v, g, lr, mu):
    w, v, g = _f64(w).copy(), _f64(v).copy(), _f64(g)
    lib().orc_sgd(_d(w), _d(v), _d(g), w.size, lr, mu)
    return w, v


# --------------------------------------------------------------------------
# the blockwise-distillation step
# --------------------------------------------------------------------------

class Oracle:
    """One teacher/student pair described by packed descriptor words."""

    def __init__(self, words, pool, batch, precision=64, momentum=0.9, eps=1e-5, rho=0.1,
                 storage=None):
        """storage="bf16": round every stored tensor to bfloat16 (see the C++ header)."""
        self._words = np.ascontiguousarray(words, dtype=np.int32)
        self._pool = np.ascontiguousarray(pool, dtype=np.float64)
        self.batch = batch
        self.B = int(self._words[2])
        self.h = lib().orc_create(self._words.ctypes.data_as(_ip), self._words.size,
                                  _d(self._pool), self._pool.size, batch, precision,
                                  momentum, eps, rho, 1 if storage == "bf16" else 0)
        if not self.h:
            raise ValueError("oracle rejected the descriptor")

    def __del__(self):
        if getattr(self, "h", None) and _lib is not None:
            _lib.orc_destroy(self.h)
            self.h = None

    def set_param(self, net, b, j, slot, arr, kind=KIND_PARAM):
        a = _f64(arr).ravel()
        if lib().orc_set_tensor(self.h, kind, net, b, j, slot, _d(a), a.size) != 0:
            raise ValueError(f"no tensor ({kind},{net},{b},{j},{slot}) of size {a.size}")

    def get_tensor(self, kind, net, b, j, slot, shape):
        out = np.empty(int(np.prod(shape)))
        if lib().orc_get_tensor(self.h, kind, net, b, j, slot, _d(out), out.size) != 0:
            raise ValueError(f"no tensor ({kind},{net},{b},{j},{slot}) of size {out.size}")
        return out.reshape(shape)

    def teacher_relay(self, x):
        """Run T_1..T_B once each; returns [A_0, ..., A_B] (flat fp64 arrays)."""
        x = _f64(x)
        lib().orc_teacher_relay(self.h, _d(x))
        acts = []
        for i in range(self.B + 1):
            a = np.empty(lib().orc_act_numel(self.h, i))
            lib().orc_get_act(self.h, i, _d(a))
            acts.append(a)
        return acts

    def teacher_upto(self, x, i):
        """A_i recomputed from the raw input through T_1..T_i."""
        x = _f64(x)
        out = np.empty(lib().orc_act_numel(self.h, i))
        lib().orc_teacher_upto(self.h, _d(x), i, _d(out))
        return out

    def student_step(self, i, a_prev, a_i, lr, mode=MODE_STEP):
        a_prev, a_i = _f64(a_prev), _f64(a_i)
        return lib().orc_student_step(self.h, i, _d(a_prev), _d(a_i), lr, mode)

    def relay_step(self, x, lr):
        x = _f64(x)
        losses = np.empty(self.B)
        lib().orc_relay_step(self.h, _d(x), lr, _d(losses))
        return losses

    def redundant_step(self, x, lr):
        x = _f64(x)
        losses = np.empty(self.B)
        lib().orc_redundant_step(self.h, _d(x), lr, _d(losses))
        return losses

    def relay_arch_step(self, x, lr):
        """Teacher once, then the architecture round (alpha trained, weights frozen) of every block."""
        x = _f64(x)
        losses = np.empty(self.B)
        lib().orc_relay_arch_step(self.h, _d(x), lr, _d(losses))
        return losses

    def set_alpha(self, b, j, alpha):
        a = _f64(alpha).ravel()
        if lib().orc_set_alpha(self.h, b, j, _d(a), a.size) != 0:
            raise ValueError(f"op {j} of block {b} is not a mix of {a.size} inputs")

    def get_alpha(self, b, j, n, kind=ALPHA_VALUE):
        out = np.empty(n)
        if lib().orc_get_alpha(self.h, kind, b, j, _d(out), n) != 0:
            raise ValueError(f"no architecture tensor {kind} for op {j} of block {b} with {n} inputs")
        return out

    def kink_margin(self, b):
        """Smallest distance of block b's last forward from a ReLU / ReLU6 / max-pool kink."""
        return lib().orc_kink_margin(self.h, b)

    SAVED_CONV, SAVED_PRE, SAVED_MEAN, SAVED_VAR = 0, 1, 2, 3

    def saved(self, b, j, which):
        """What the last forward of student block b kept for op j: the convolution output, the tensor
        before the activation, the batch mean or the biased batch variance."""
        n = lib().orc_saved_numel(self.h, b, j, which)
        if n < 0:
            raise ValueError("no such saved tensor")
        out = np.empty(n)
        lib().orc_get_saved(self.h, b, j, which, _d(out))
        return out

    def value(self, b, v):
        n = lib().orc_value_numel(self.h, b, v)
        if n < 0:
            raise ValueError("no such value")
        out = np.empty(n)
        lib().orc_get_value(self.h, b, v, _d(out))
        return out
