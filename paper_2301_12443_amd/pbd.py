"""ctypes binding over libpbd.so: same names as include/pbd.h, argument
marshalling only.  PyTorch supplies device memory and the stream; every step of
the path runs in the library's HIP kernels.  There is no fallback: if the
library is missing, loading raises."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import workloads as W

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpbd.so")

PBD_F32, PBD_BF16 = 0, 1
PBD_TEACHER, PBD_STUDENT = 0, 1
PBD_PARAM, PBD_GRAD, PBD_MOMENTUM, PBD_PROB = 0, 1, 2, 3
STATUS = {0: "PBD_OK", -1: "PBD_EINVAL", -2: "PBD_ESHAPE", -3: "PBD_ENOMEM_WS",
          -4: "PBD_ESTATE", -5: "PBD_EHIP"}

SYMBOLS = ["pbd_create", "pbd_destroy", "pbd_last_error", "pbd_num_blocks", "pbd_workspace_bytes",
           "pbd_bind", "pbd_load_param", "pbd_read_tensor", "pbd_read_act", "pbd_read_value",
           "pbd_read_conv_out", "pbd_read_batch_stats", "pbd_read_grad_value",
           "pbd_teacher_relay", "pbd_teacher_prefix", "pbd_student_step", "pbd_student_step_static", "pbd_distill_step", "pbd_pipeline_step", "pbd_pipeline_flush", "pbd_set_pipeline_order", "pbd_uses_graph", "pbd_sync",
           "pbd_arch_step", "pbd_distill_arch_step", "pbd_load_alpha", "pbd_read_alpha",
           "pbd_set_profile", "pbd_reset_profile", "pbd_get_profile"]


class pbd_opts(C.Structure):
    _fields_ = [("batch", C.c_int32), ("precision", C.c_int32), ("momentum", C.c_float),
                ("bn_eps", C.c_float), ("bn_momentum", C.c_float), ("force_direct", C.c_int32), ("no_graph", C.c_int32)]


class pbd_tensor(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("n", C.c_int32), ("c", C.c_int32), ("h", C.c_int32),
                ("w", C.c_int32), ("c_phys", C.c_int32), ("dtype", C.c_int32)]


class pbd_prof_entry(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("ms", C.c_float), ("bytes", C.c_double),
                ("flops", C.c_double), ("net", C.c_int32), ("block", C.c_int32), ("op", C.c_int32)]


class PbdError(RuntimeError):
    def __init__(self, code, msg=""):
        super().__init__(f"{STATUS.get(code, code)}: {msg}")
        self.code = code


_lib = None


def lib():
    """Load libpbd.so; raises if it has not been built (python -m paper_2301_12443_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with "
                                    "`python -m paper_2301_12443_amd.build`; there is no fallback path")
        L = C.CDLL(LIB_PATH)
        fp, ip, dp = C.POINTER(C.c_float), C.POINTER(C.c_int32), C.POINTER(C.c_double)
        L.pbd_create.argtypes = [ip, C.c_int32, dp, C.c_int32, C.POINTER(pbd_opts), C.POINTER(C.c_void_p)]
        L.pbd_destroy.argtypes = [C.c_void_p]
        L.pbd_destroy.restype = None
        L.pbd_last_error.argtypes = [C.c_void_p]
        L.pbd_last_error.restype = C.c_char_p
        L.pbd_num_blocks.argtypes = [C.c_void_p]
        L.pbd_workspace_bytes.argtypes = [C.c_void_p]
        L.pbd_workspace_bytes.restype = C.c_size_t
        L.pbd_bind.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.pbd_load_param.argtypes = [C.c_void_p] + [C.c_int32] * 4 + [fp, C.c_size_t]
        L.pbd_read_tensor.argtypes = [C.c_void_p] + [C.c_int32] * 5 + [fp, C.c_size_t]
        L.pbd_read_act.argtypes = [C.c_void_p, C.c_int32, fp, C.c_size_t]
        L.pbd_read_value.argtypes = [C.c_void_p, C.c_int32, C.c_int32, fp, C.c_size_t]
        L.pbd_read_conv_out.argtypes = [C.c_void_p, C.c_int32, C.c_int32, fp, C.c_size_t]
        L.pbd_read_batch_stats.argtypes = [C.c_void_p, C.c_int32, C.c_int32, fp, fp, C.c_size_t]
        L.pbd_read_grad_value.argtypes = [C.c_void_p, C.c_int32, C.c_int32, fp, C.c_size_t]
        L.pbd_teacher_relay.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(pbd_tensor)]
        L.pbd_teacher_prefix.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(pbd_tensor)]
        L.pbd_student_step.argtypes = [C.c_void_p, C.c_int32, C.POINTER(pbd_tensor), C.POINTER(pbd_tensor),
                                       C.c_float, C.c_void_p]
        L.pbd_distill_step.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_void_p]
        L.pbd_arch_step.argtypes = L.pbd_student_step.argtypes
        L.pbd_student_step_static.argtypes = L.pbd_student_step.argtypes
        L.pbd_distill_arch_step.argtypes = L.pbd_distill_step.argtypes
        L.pbd_pipeline_step.argtypes = L.pbd_distill_step.argtypes
        L.pbd_pipeline_flush.argtypes = [C.c_void_p, C.c_void_p]
        L.pbd_set_pipeline_order.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_int32]
        L.pbd_load_alpha.argtypes = [C.c_void_p, C.c_int32, C.c_int32, fp, C.c_size_t]
        L.pbd_read_alpha.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, fp, C.c_size_t]
        L.pbd_uses_graph.argtypes = [C.c_void_p]
        L.pbd_sync.argtypes = [C.c_void_p]
        L.pbd_set_profile.argtypes = [C.c_void_p, C.c_int32]
        L.pbd_reset_profile.argtypes = [C.c_void_p]
        L.pbd_get_profile.argtypes = [C.c_void_p, C.POINTER(pbd_prof_entry), C.c_int32]
        _lib = L
    return _lib


def _fp(a):
    return a.ctypes.data_as(C.POINTER(C.c_float))


class Distiller:
    """A context for one workload.  `create` needs no GPU; `bind` and everything after do."""

    def __init__(self, wl: W.Workload, batch: int | None = None, precision: str | None = None,
                 force_direct: bool = False, bn_eps: float = 1e-5, bn_momentum: float = 0.1,
                 no_graph: bool = False):
        self.wl = wl
        self.batch = wl.batch if batch is None else batch
        self.precision = PBD_BF16 if (precision or wl.precision) == "bf16" else PBD_F32
        self.B = wl.B
        words, pool = W.pack(wl)
        self._words, self._pool = words, pool
        opts = pbd_opts(self.batch, self.precision, wl.momentum, bn_eps, bn_momentum, int(force_direct),
                        int(no_graph))
        h = C.c_void_p()
        rc = lib().pbd_create(words.ctypes.data_as(C.POINTER(C.c_int32)), words.size,
                              pool.ctypes.data_as(C.POINTER(C.c_double)), pool.size, C.byref(opts), C.byref(h))
        if rc != 0:
            raise PbdError(rc, lib().pbd_last_error(None).decode())
        self.h = h
        self._ws = None
        self.views = None
        self.act_shapes = W.activation_shapes(wl)

    def __del__(self):
        if getattr(self, "h", None) and _lib is not None:   # (module globals are gone at interpreter exit)
            _lib.pbd_destroy(self.h)
            self.h = None

    def _check(self, rc):
        if rc < 0:
            raise PbdError(rc, lib().pbd_last_error(self.h).decode())
        return rc

    def workspace_bytes(self) -> int:
        return lib().pbd_workspace_bytes(self.h)

    def bind(self, device="cuda:0", stream=None):
        import torch
        self.device = torch.device(device)
        self._ws = torch.empty(self.workspace_bytes() + 256, dtype=torch.uint8, device=self.device)
        base = (self._ws.data_ptr() + 255) // 256 * 256
        # a stream of its own (not the legacy default stream) so that the library can capture the
        # step into a HIP graph; callers order against it with sync() or stream events
        self._stream = stream if stream is not None else torch.cuda.Stream(self.device)
        self.losses = torch.zeros(self.B, dtype=torch.float32, device=self.device)
        torch.cuda.synchronize(self.device)
        self._check(lib().pbd_bind(self.h, base, self.workspace_bytes(), self._stream.cuda_stream))
        return self

    def load_params(self):
        """Seeded parameters of both nets (He-normal weights, frozen teacher BN, identity student BN)."""
        for net, b, j, slot, arr in W.iter_params(self.wl):
            self.load_param(net, b, j, slot, arr)

    def load_param(self, net, b, j, slot, arr):
        a = np.ascontiguousarray(arr, dtype=np.float32).ravel()
        self._check(lib().pbd_load_param(self.h, net, b, j, slot, _fp(a), a.size))

    def read_tensor(self, kind, net, b, j, slot, shape):
        out = np.empty(int(np.prod(shape)), dtype=np.float32)
        self._check(lib().pbd_read_tensor(self.h, kind, net, b, j, slot, _fp(out), out.size))
        return out.reshape(shape)

    def read_act(self, i):
        shape = (self.batch, *self.act_shapes[i])
        out = np.empty(int(np.prod(shape)), dtype=np.float32)
        self._check(lib().pbd_read_act(self.h, i, _fp(out), out.size))
        return out.reshape(shape)

    def read_value(self, b, v):
        shape = (self.batch, *W.block_shapes(self.wl.student[b], self.act_shapes[b])[v])
        out = np.empty(int(np.prod(shape)), dtype=np.float32)
        self._check(lib().pbd_read_value(self.h, b, v, _fp(out), out.size))
        return out.reshape(shape)

    def read_conv_out(self, b, j):
        """Output of the convolution of student op j of block b (before normalisation), float32 NCHW."""
        shape = (self.batch, *W.block_shapes(self.wl.student[b], self.act_shapes[b])[j + 1])
        out = np.empty(int(np.prod(shape)), dtype=np.float32)
        self._check(lib().pbd_read_conv_out(self.h, b, j, _fp(out), out.size))
        return out.reshape(shape)

    def read_batch_stats(self, b, j):
        """(batch mean, 1 / sqrt(biased batch variance + eps)) of student op j of block b."""
        n = W.block_shapes(self.wl.student[b], self.act_shapes[b])[j + 1][0]
        mean, invstd = np.empty(n, dtype=np.float32), np.empty(n, dtype=np.float32)
        self._check(lib().pbd_read_batch_stats(self.h, b, j, _fp(mean), _fp(invstd), n))
        return mean, invstd

    def read_grad_value(self, b, v):
        """The stored gradient that belongs to value v of block b (see pbd_read_grad_value)."""
        shape = (self.batch, *W.block_shapes(self.wl.student[b], self.act_shapes[b])[v])
        out = np.empty(int(np.prod(shape)), dtype=np.float32)
        self._check(lib().pbd_read_grad_value(self.h, b, v, _fp(out), out.size))
        return out.reshape(shape)

    def _check_x(self, x_dev):
        """The C ABI takes a bare device pointer for x and reads batch * C0 * H0 * W0 float32 from it, so
        everything it cannot check is checked here, before any launch: a float32, contiguous tensor of shape
        (batch, C0, H0, W0) on the device the context is bound to."""
        import torch
        if self._ws is None:
            raise PbdError(-4, "no workspace bound (call bind first)")
        want = (self.batch, *self.wl.in_shape)
        if not isinstance(x_dev, torch.Tensor):
            raise PbdError(-1, f"x must be a torch tensor, got {type(x_dev).__name__}")
        if x_dev.dtype != torch.float32:
            raise PbdError(-1, f"x must be float32, got {x_dev.dtype}")
        if tuple(x_dev.shape) != want:
            raise PbdError(-2, f"x must have shape {want}, got {tuple(x_dev.shape)}")
        if not x_dev.is_contiguous():
            raise PbdError(-1, "x must be contiguous (NCHW)")
        if not x_dev.is_cuda or x_dev.device != self._ws.device:
            raise PbdError(-1, f"x must live on {self._ws.device}, got {x_dev.device}")
        return x_dev.data_ptr()

    def teacher_relay(self, x_dev):
        """x_dev: float32 NCHW CUDA tensor.  Returns the B+1 borrowed views A_0..A_B."""
        self._check_x(x_dev)
        views = (pbd_tensor * (self.B + 1))()
        self._check(lib().pbd_teacher_relay(self.h, x_dev.data_ptr(), views))
        self.views = views
        return views

    def teacher_prefix(self, x_dev, upto):
        """The teacher without relaying: T_1..T_upto from x.  Returns the views A_0..A_upto."""
        self._check_x(x_dev)
        views = (pbd_tensor * (self.B + 1))()
        self._check(lib().pbd_teacher_prefix(self.h, x_dev.data_ptr(), upto, views))
        self.views = views
        return views

    def student_step(self, i, lr, a_prev=None, a_i=None):
        """Block i (1-based).  The loss lands in self.losses[i-1] on the device."""
        a_prev = self.views[i - 1] if a_prev is None else a_prev
        a_i = self.views[i] if a_i is None else a_i
        self._check(lib().pbd_student_step(self.h, i, C.byref(a_prev), C.byref(a_i), lr,
                                           self.losses.data_ptr() + 4 * (i - 1)))

    def student_step_static(self, i, lr, a_prev=None, a_i=None):
        """student_step with the reduction scratch in the library's static device array (allocates nothing)."""
        a_prev = self.views[i - 1] if a_prev is None else a_prev
        a_i = self.views[i] if a_i is None else a_i
        self._check(lib().pbd_student_step_static(self.h, i, C.byref(a_prev), C.byref(a_i), lr,
                                                  self.losses.data_ptr() + 4 * (i - 1)))

    def distill_step(self, x_dev, lr):
        self._check(lib().pbd_distill_step(self.h, self._check_x(x_dev), lr, self.losses.data_ptr()))

    def pipeline_step(self, x_dev, lr):
        """Hand in a batch: the teacher relays it while the students train on the batch before."""
        self._check(lib().pbd_pipeline_step(self.h, self._check_x(x_dev), lr, self.losses.data_ptr()))

    def pipeline_flush(self):
        self._check(lib().pbd_pipeline_flush(self.h, self.losses.data_ptr()))

    def set_pipeline_order(self, order):
        """Capture order of the pipelined step's branches: a permutation of 0..B (B = the teacher)."""
        arr = (C.c_int32 * len(order))(*order)
        self._check(lib().pbd_set_pipeline_order(self.h, arr, len(order)))

    def arch_step(self, i, lr_alpha, a_prev=None, a_i=None):
        """Architecture round of block i (1-based): alpha trained, weights frozen."""
        a_prev = self.views[i - 1] if a_prev is None else a_prev
        a_i = self.views[i] if a_i is None else a_i
        self._check(lib().pbd_arch_step(self.h, i, C.byref(a_prev), C.byref(a_i), lr_alpha,
                                        self.losses.data_ptr() + 4 * (i - 1)))

    def distill_arch_step(self, x_dev, lr_alpha):
        self._check(lib().pbd_distill_arch_step(self.h, self._check_x(x_dev), lr_alpha, self.losses.data_ptr()))

    def load_alpha(self, b, j, alpha):
        a = np.ascontiguousarray(alpha, dtype=np.float32).ravel()
        self._check(lib().pbd_load_alpha(self.h, b, j, _fp(a), a.size))

    def read_alpha(self, b, j, n, kind=PBD_PARAM):
        out = np.empty(n, dtype=np.float32)
        self._check(lib().pbd_read_alpha(self.h, kind, b, j, _fp(out), n))
        return out

    def uses_graph(self) -> bool:
        return bool(lib().pbd_uses_graph(self.h))

    def sync(self):
        self._check(lib().pbd_sync(self.h))

    def set_profile(self, on: bool):
        self._check(lib().pbd_set_profile(self.h, int(on)))

    def reset_profile(self):
        self._check(lib().pbd_reset_profile(self.h))

    def get_profile(self):
        n = self._check(lib().pbd_get_profile(self.h, None, 0))
        buf = (pbd_prof_entry * max(n, 1))()
        self._check(lib().pbd_get_profile(self.h, buf, n))
        return [dict(name=e.name.decode(), ms=e.ms, bytes=e.bytes, flops=e.flops,
                     net=e.net, block=e.block, op=e.op) for e in buf[:n]]
