"""Steps pipelined over batches (Sec. IV-A teacher relaying, Sec. IV-B decoupled updates): the teacher
relays batch k while the students train on batch k-1.  The schedule changes, the arithmetic does not:
K pipelined calls and a flush must leave, bit for bit, what K whole steps leave - and those are the
steps the other GPU tests hold against the oracle."""
import numpy as np
import pytest

from helpers import make_oracle, max_rel, pattern_workloads
from paper_2301_12443_amd import pbd, workloads as W

pytestmark = pytest.mark.gpu


def _distiller(wl, precision, no_graph=False):
    d = pbd.Distiller(wl, precision=precision, no_graph=no_graph)
    d.bind("cuda:0")
    d.load_params()
    return d


def _state(d, wl):
    out = {}
    for b in range(wl.B):
        for (j, slot), shape in W.param_shapes(wl, W.NET_STUDENT, b).items():
            for kind in (pbd.PBD_PARAM, pbd.PBD_MOMENTUM, pbd.PBD_GRAD):
                if kind != pbd.PBD_PARAM and slot in (W.P_RMEAN, W.P_RVAR):
                    continue
                out[(b, j, slot, kind)] = d.read_tensor(kind, 1, b, j, slot, shape)
    return out


def _batches(wl, k):
    import torch
    return [torch.from_numpy(W.make_input(wl, step=s)).cuda() for s in range(k)]


CASES = [W.tiny_cnn()] + pattern_workloads()


@pytest.mark.parametrize("wl", CASES, ids=[w.name for w in CASES])
@pytest.mark.parametrize("precision", ["f32", "bf16"])
@pytest.mark.parametrize("no_graph", [False, True], ids=["graph", "direct"])
def test_pipelined_steps_equal_whole_steps_bit_for_bit(wl, precision, no_graph):
    k = 5
    xs = _batches(wl, k)
    lrs = [wl.lr * (1.0 - 0.1 * s) for s in range(k)]
    plain, piped = _distiller(wl, precision, no_graph), _distiller(wl, precision, no_graph)
    want_losses, got_losses = [], []
    for x, lr in zip(xs, lrs):
        plain.distill_step(x, lr)
        plain.sync()
        want_losses.append(plain.losses.cpu().numpy().copy())
    for s, (x, lr) in enumerate(zip(xs, lrs)):
        piped.pipeline_step(x, lr)
        piped.sync()
        if s:
            got_losses.append(piped.losses.cpu().numpy().copy())
    assert piped.uses_graph() == (not no_graph)
    # the batch in flight is the one the views show
    assert np.array_equal(piped.read_act(wl.B), plain.read_act(wl.B))
    piped.pipeline_flush()
    piped.sync()
    got_losses.append(piped.losses.cpu().numpy().copy())
    assert np.array_equal(np.array(got_losses), np.array(want_losses))
    a, b = _state(plain, wl), _state(piped, wl)
    for key in a:
        assert np.array_equal(a[key], b[key]), key
    # after the flush the one-step calls work again, and both go on alike
    plain.distill_step(xs[0], wl.lr)
    piped.distill_step(xs[0], wl.lr)
    plain.sync(); piped.sync()
    assert np.array_equal(plain.losses.cpu().numpy(), piped.losses.cpu().numpy())


def test_pipelined_steps_against_the_oracle():
    """Three batches through the pipeline against three steps of the fp64 oracle."""
    wl = W.tiny_cnn()
    k = 3
    xs = [W.make_input(wl, step=s) for s in range(k)]
    o = make_oracle(wl)
    want = [o.relay_step(x, wl.lr) for x in xs]
    d = _distiller(wl, "f32")
    import torch
    got = []
    for s, x in enumerate(xs):
        d.pipeline_step(torch.from_numpy(x).cuda(), wl.lr)
        d.sync()
        if s:
            got.append(d.losses.cpu().numpy().copy())
    d.pipeline_flush(); d.sync()
    got.append(d.losses.cpu().numpy().copy())
    assert max_rel(np.array(got), np.array(want)) < 1e-4
    for b in range(wl.B):
        for (j, slot), shape in W.param_shapes(wl, W.NET_STUDENT, b).items():
            assert max_rel(d.read_tensor(pbd.PBD_PARAM, 1, b, j, slot, shape),
                           o.get_tensor(0, 1, b, j, slot, shape)) < 1e-4, (b, j, slot)


def test_calls_that_do_not_mix_with_a_batch_in_flight():
    import torch
    wl = W.tiny_cnn()
    d = _distiller(wl, "f32")
    x = torch.from_numpy(W.make_input(wl)).cuda()
    d.pipeline_flush()                       # nothing waits: no-op
    d.pipeline_step(x, wl.lr)
    for call in (lambda: d.distill_step(x, wl.lr), lambda: d.teacher_relay(x), lambda: d.teacher_prefix(x, 1)):
        with pytest.raises(pbd.PbdError) as e:
            call()
        assert e.value.code == -4          # PBD_ESTATE
    with pytest.raises(pbd.PbdError):
        d.read_value(0, 1)                   # the students hold the values of no batch yet
    with pytest.raises(pbd.PbdError):
        d.pipeline_step(x, float("nan"))
    d.pipeline_flush(); d.sync()
    d.read_value(0, 1)
    d.distill_step(x, wl.lr); d.sync()


def test_full_size_pipelined_steps_equal_whole_steps():
    """Configuration 2 at its full batch, in the launch configuration the benchmark times (graph replay of
    the pipelined body): four batches leave bit for bit the losses, weights, momenta and running statistics
    of four whole steps - and the whole step at this size is held against the oracle elsewhere."""
    wl = W.vgg16_dsconv()
    k = 4
    xs = _batches(wl, k)
    plain, piped = _distiller(wl, None), _distiller(wl, None)
    want, got = [], []
    for x in xs:
        plain.distill_step(x, wl.lr)
        plain.sync()
        want.append(plain.losses.cpu().numpy().copy())
    for s, x in enumerate(xs):
        piped.pipeline_step(x, wl.lr)
        piped.sync()
        if s:
            got.append(piped.losses.cpu().numpy().copy())
    piped.pipeline_flush()
    piped.sync()
    got.append(piped.losses.cpu().numpy().copy())
    assert piped.uses_graph()
    assert np.array_equal(np.array(got), np.array(want))
    for i in range(wl.B + 1):
        assert np.array_equal(piped.read_act(i), plain.read_act(i)), i
    a, b = _state(plain, wl), _state(piped, wl)
    for key in a:
        assert np.array_equal(a[key], b[key]), key


def test_capture_order_of_the_branches_changes_no_bit():
    """The branches of the pipelined step are independent (Sec. IV-B): whatever order they are captured in,
    the losses and the trained state are the same bits."""
    wl = pattern_workloads()[0]
    k = 3
    xs = _batches(wl, k)
    ref = None
    B = wl.B
    for order in (None, list(range(B, -1, -1)), [B] + list(range(B)), list(range(B - 1, -1, -1)) + [B]):
        d = _distiller(wl, "bf16")
        if order is not None:
            d.set_pipeline_order(order)
        losses = []
        for s, x in enumerate(xs):
            d.pipeline_step(x, wl.lr)
            d.sync()
            if s:
                losses.append(d.losses.cpu().numpy().copy())
            if s == 0 and order is not None:
                with pytest.raises(pbd.PbdError):      # not while a batch waits
                    d.set_pipeline_order(order)
        d.pipeline_flush(); d.sync()
        losses.append(d.losses.cpu().numpy().copy())
        assert d.uses_graph()
        got = (np.array(losses), _state(d, wl))
        if ref is None:
            ref = got
        else:
            assert np.array_equal(got[0], ref[0]), order
            for key in ref[1]:
                assert np.array_equal(got[1][key], ref[1][key]), (order, key)
    d = _distiller(wl, "bf16")
    for bad in ([0] * (B + 1), list(range(B)), list(range(1, B + 2))):
        with pytest.raises(pbd.PbdError):
            d.set_pipeline_order(bad)
    # a new order after graphs exist: captured again, same bits as before
    d.pipeline_step(xs[0], wl.lr); d.pipeline_step(xs[1], wl.lr); d.pipeline_flush(); d.sync()
    d.set_pipeline_order(list(range(B, -1, -1)))
    d.pipeline_step(xs[2], wl.lr); d.pipeline_flush(); d.sync()
    assert np.array_equal(d.losses.cpu().numpy(), ref[0][-1])
