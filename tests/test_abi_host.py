"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares,
and validates descriptors and options without touching a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2301_12443_amd import pbd, workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "pbd.h")).read()
    declared = set(re.findall(r"\b(pbd_[a-z_]+)\s*\(", header))
    assert declared == set(pbd.SYMBOLS)
    L = pbd.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_struct_layouts_match_header():
    assert C.sizeof(pbd.pbd_opts) == 28
    assert C.sizeof(pbd.pbd_tensor) == 32
    assert C.sizeof(pbd.pbd_prof_entry) == 72


def _create(words, pool, opts):
    h = C.c_void_p()
    rc = pbd.lib().pbd_create(words.ctypes.data_as(C.POINTER(C.c_int32)), words.size,
                              pool.ctypes.data_as(C.POINTER(C.c_double)), pool.size, C.byref(opts), C.byref(h))
    if h:
        pbd.lib().pbd_destroy(h)
    return rc, pbd.lib().pbd_last_error(None).decode()


def test_create_validates_descriptor_and_options():
    wl = W.tiny_cnn()
    words, pool = W.pack(wl)
    ok = pbd.pbd_opts(8, pbd.PBD_F32, 0.9, 1e-5, 0.1, 0)
    assert _create(words, pool, ok)[0] == 0
    bad = words.copy(); bad[0] = 7
    assert _create(bad, pool, ok)[0] == -2
    assert _create(words[:40], pool, ok)[0] == -2                       # truncated
    bad = words.copy(); bad[6 + 1 + 10] = 12                            # teacher op 0: C_out 16 -> 12
    rc, msg = _create(bad, pool, ok)
    assert rc == -2 and "C_out" in msg
    bad = words.copy(); bad[6 + 1 + 2] = 3                              # input refers forward
    assert _create(bad, pool, ok)[0] == -2
    for o in (pbd.pbd_opts(0, 0, 0.9, 1e-5, 0.1, 0), pbd.pbd_opts(8, 2, 0.9, 1e-5, 0.1, 0),
              pbd.pbd_opts(8, 0, 1.5, 1e-5, 0.1, 0), pbd.pbd_opts(8, 0, 0.9, 0.0, 0.1, 0),
              pbd.pbd_opts(8, 0, float("nan"), 1e-5, 0.1, 0)):
        assert _create(words, pool, o)[0] == -1
    # teacher and student of a pair must produce the same shape (Sec. II-A)
    t, s = W.Block(), W.Block()
    t.cba(0, 16, 3); s.cba(0, 16, 3, 2)
    w2 = W.Workload("bad", 2, (3, 8, 8), [t], [s], "f32", lr=0.1)
    with pytest.raises(AssertionError):
        W.pack(w2)


def test_create_rejects_degenerate_and_oversized_shapes():
    """Limits of the kernels, enforced on the host before anything is launched."""
    # a single block with a single op per net on a 1x1 image is a complete workload at batch 2 ...
    t, s = W.Block(), W.Block()
    t.cba(0, 8, 1); s.cba(0, 8, 1)
    one = W.Workload("one", 2, (8, 1, 1), [t], [s], "f32", lr=0.1)
    words, pool = W.pack(one)
    assert _create(words, pool, pbd.pbd_opts(2, pbd.PBD_F32, 0.9, 1e-5, 0.1, 0))[0] == 0
    # ... but at batch 1 the student's batch norm would see one value per channel
    rc, msg = _create(words, pool, pbd.pbd_opts(1, pbd.PBD_F32, 0.9, 1e-5, 0.1, 0))
    assert rc == -2 and "one value per channel" in msg
    # 32-bit byte offsets: a tensor must stay below 2 GiB (ResNet-50 x1.5 at batch 1500, bf16: 2.2 GiB in block 1)
    wl = W.resnet50_wide(batch=1500)
    words, pool = W.pack(wl)
    rc, msg = _create(words, pool, pbd.pbd_opts(1500, pbd.PBD_BF16, 0.9, 1e-5, 0.1, 0))
    assert rc == -2 and "2 GiB" in msg
    assert _create(words, pool, pbd.pbd_opts(256, pbd.PBD_BF16, 0.9, 1e-5, 0.1, 0))[0] == 0


def test_workspace_sizes_and_unbound_calls():
    for name, make in W.CONFIGS.items():
        d = pbd.Distiller(make())
        assert d.workspace_bytes() > 0 and d.workspace_bytes() < 200 * 2**30   # fits 288 GB of HBM
        assert pbd.lib().pbd_num_blocks(d.h) == make().B
    d = pbd.Distiller(W.tiny_cnn())
    buf = np.zeros(4, dtype=np.float32)
    assert pbd.lib().pbd_load_param(d.h, 0, 0, 0, 0, buf.ctypes.data_as(C.POINTER(C.c_float)), 4) == -4
    assert b"pbd_bind" in pbd.lib().pbd_last_error(d.h)
    assert pbd.lib().pbd_distill_step(d.h, None, 0.1, None) == -4
    assert pbd.lib().pbd_sync(None) == -1


def test_binding_rejects_a_wrong_input_tensor_before_any_launch():
    """The ABI carries no size for x_dev (a bare device pointer to batch x C0 x H0 x W0 float32), so the
    binding checks dtype, shape, device and contiguity itself and raises before the library is called."""
    import torch
    wl = W.tiny_cnn()
    d = pbd.Distiller(wl)
    with pytest.raises(pbd.PbdError, match="PBD_ESTATE"):
        d.distill_step(torch.zeros(8, 3, 32, 32), wl.lr)
    d._ws = torch.empty(1, dtype=torch.uint8)        # stands in for a bound workspace (no GPU here)
    d.losses = torch.zeros(wl.B)
    good = torch.zeros(wl.batch, *wl.in_shape, dtype=torch.float32)
    calls = [lambda x: d.teacher_relay(x), lambda x: d.teacher_prefix(x, 1), lambda x: d.distill_step(x, wl.lr),
             lambda x: d.pipeline_step(x, wl.lr), lambda x: d.distill_arch_step(x, 0.01)]
    for call in calls:
        with pytest.raises(pbd.PbdError, match="float32"):
            call(good.to(torch.bfloat16))
        with pytest.raises(pbd.PbdError, match="float32"):
            call(good.double())
        with pytest.raises(pbd.PbdError, match="shape"):
            call(good[:4])
        with pytest.raises(pbd.PbdError, match="shape"):
            call(good.reshape(wl.batch, -1))
        with pytest.raises(pbd.PbdError, match="contiguous"):
            call(torch.zeros(wl.batch, wl.in_shape[0], wl.in_shape[1], 2 * wl.in_shape[2])[..., ::2])
        with pytest.raises(pbd.PbdError, match="must live on"):
            call(good)                                # a host tensor
        with pytest.raises(pbd.PbdError, match="torch tensor"):
            call(np.zeros((wl.batch, *wl.in_shape), dtype=np.float32))
    d._ws = None
