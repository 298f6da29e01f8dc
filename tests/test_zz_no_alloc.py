"""pbd_student_step_static, the variant of pbd_student_step for callers that cannot allocate: its reduction
scratch is a static device array inside the library.  Called through the C ABI and compared with
pbd_student_step on a twin context, bit for bit (same kernels, same order of every sum), on two calls in a
row, the second on a smaller block, so that whatever the first call left in the shared array is in place
when the second one runs."""
import ctypes as C

import numpy as np
import pytest

import parity
from helpers import layer_workloads
from paper_2301_12443_amd import pbd, workloads as W

pytestmark = pytest.mark.gpu


def _state(d, wl, b):
    out = {}
    for (j, slot), shape in W.param_shapes(wl, W.NET_STUDENT, b).items():
        out[(j, slot, "param")] = d.read_tensor(pbd.PBD_PARAM, 1, b, j, slot, shape).copy()
        if slot <= W.P_BETA:
            out[(j, slot, "grad")] = d.read_tensor(pbd.PBD_GRAD, 1, b, j, slot, shape).copy()
            out[(j, slot, "mom")] = d.read_tensor(pbd.PBD_MOMENTUM, 1, b, j, slot, shape).copy()
    return out


def _value(d, b, v):
    """Saved value v of block b, or None where the library does not keep it (its reader applies the normalisation)."""
    try:
        return d.read_value(b, v)
    except pbd.PbdError as e:
        if e.code != -4:
            raise
        return None


@pytest.mark.parametrize("precision,batch", [("f32", 8), ("bf16", 8), ("bf16", 96)])
def test_static_scratch_step_equals_the_workspace_step(precision, batch):
    import torch
    L = pbd.lib()
    wl = W.tiny_cnn()
    x = torch.from_numpy(W.make_input(wl, batch=batch)).cuda()
    ref = parity.make_distiller(wl, batch=batch, precision=precision)
    dut = parity.make_distiller(wl, batch=batch, precision=precision)
    ref.teacher_relay(x)
    views = dut.teacher_relay(x)
    # block 1 (32 x 32 images: the largest tensors and partial sums), then block 4 (4 x 4 images)
    for step, i in enumerate((1, 4, 2)):
        ref.student_step(i, wl.lr)
        ref.sync()
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        rc = L.pbd_student_step_static(dut.h, i, C.byref(views[i - 1]), C.byref(views[i]), wl.lr,
                                       dut.losses.data_ptr() + 4 * (i - 1))
        assert rc == 0, L.pbd_last_error(dut.h)
        dut.sync()
        assert torch.cuda.mem_get_info()[0] == free_before, "the call changed the amount of free device memory"
        assert dut.losses[i - 1].item() == ref.losses[i - 1].item()
        assert np.isfinite(dut.losses[i - 1].item()) and dut.losses[i - 1].item() > 0
        a, b = _state(ref, wl, i - 1), _state(dut, wl, i - 1)
        for k in a:
            np.testing.assert_array_equal(a[k], b[k], err_msg=f"call {step}, block {i}, tensor {k}")
        for v in range(1, len(wl.student[i - 1].ops) + 1):
            want, got = _value(ref, i - 1, v), _value(dut, i - 1, v)
            assert (want is None) == (got is None)
            if want is not None:
                np.testing.assert_array_equal(want, got)
    # a second step of block 1 on both sides: momentum in play, the array now holds block 2's leftovers
    ref.student_step(1, wl.lr); ref.sync()
    dut.student_step_static(1, wl.lr); dut.sync()
    a, b = _state(ref, wl, 0), _state(dut, wl, 0)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])


def test_static_scratch_step_rejects_what_does_not_fit_and_bad_arguments():
    import torch
    L = pbd.lib()
    wl = [c for c in layer_workloads() if c[0].name == "l_deepK3x3"][0][0]
    batch = 256       # 12544 pixels: the weight gradient of the 3 x 3 layer is cut into several pixel ranges
    d = parity.make_distiller(wl, batch=batch, precision="bf16")
    x = torch.from_numpy(W.make_input(wl, batch=batch)).cuda()
    loss = torch.zeros(1, device="cuda")
    v = pbd.pbd_tensor()
    assert L.pbd_student_step_static(d.h, 1, C.byref(v), C.byref(v), 0.1, loss.data_ptr()) == -4     # no relay yet
    views = d.teacher_relay(x)
    before = d.read_tensor(pbd.PBD_PARAM, 1, 0, 1, W.P_WEIGHT, (384, 384, 3, 3)).copy()
    # partial weight gradients of 384 x 3456 floats (5.3 MB) for each of four or more pixel ranges: more than the
    # 16 MiB array holds
    rc = L.pbd_student_step_static(d.h, 1, C.byref(views[0]), C.byref(views[1]), 0.1, loss.data_ptr())
    assert rc == -3 and b"static" in L.pbd_last_error(d.h)
    d.sync()
    np.testing.assert_array_equal(before, d.read_tensor(pbd.PBD_PARAM, 1, 0, 1, W.P_WEIGHT, (384, 384, 3, 3)))
    assert L.pbd_student_step_static(d.h, 0, C.byref(views[0]), C.byref(views[1]), 0.1, loss.data_ptr()) == -1
    assert L.pbd_student_step_static(d.h, 1, C.byref(views[1]), C.byref(views[1]), 0.1, loss.data_ptr()) == -2
    assert L.pbd_student_step_static(d.h, 1, C.byref(views[0]), C.byref(views[1]), float("inf"), loss.data_ptr()) == -1
    assert L.pbd_student_step_static(d.h, 1, C.byref(views[0]), C.byref(views[1]), 0.1, None) == -1
    d.set_profile(True)
    assert L.pbd_student_step_static(d.h, 1, C.byref(views[0]), C.byref(views[1]), 0.1, loss.data_ptr()) == -4
    d.set_profile(False)
    d.student_step(1, 0.1)      # the workspace form has no such limit
    d.sync()
    assert np.isfinite(d.losses[0].item())
