"""Pins for the two parts of the oracle that the bf16 comparisons lean on and that the whole-step pins
do not reach: the bfloat16 storage rounding (against the CPU library's float32 -> bfloat16 conversion,
plus ties, subnormals and non-finite values by hand), where exactly the storage mode applies it (each
stored tensor and nothing else), and the kink-margin diagnostic on hand-built cases whose margin is
known in closed form."""
import numpy as np
import pytest
import torch

from helpers import make_oracle
from oracle import pbd_oracle as orc
from paper_2301_12443_amd import workloads as W


def _is_bf16(a):
    """True where a (float64 array) is exactly representable in bfloat16."""
    f = np.asarray(a, dtype=np.float64)
    f32 = f.astype(np.float32)
    return (f32.astype(np.float64) == f) & ((f32.view(np.uint32) & 0xffff) == 0)


# ---------------------------------------------------------------------------
# round_bf16
# ---------------------------------------------------------------------------

def test_round_bf16_equals_the_library_conversion_on_random_values():
    """Values of every magnitude a step produces (1e-30 .. 1e30, both signs), exactly representable in
    float32, against torch's float32 -> bfloat16 cast, which rounds to nearest even."""
    g = np.random.default_rng(11)
    x = (g.standard_normal(400000) * np.exp(g.uniform(-70, 70, 400000))).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    got = orc.round_bf16(x.astype(np.float64))
    np.testing.assert_array_equal(got, want)
    # every float32 bit pattern of one binade (mantissa sweep): all 65536 low halves, both rounding directions
    bits = (np.uint32(0x3f800000) + np.arange(1 << 18, dtype=np.uint32) * np.uint32(32)).view(np.float32)
    want = torch.from_numpy(bits.copy()).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(orc.round_bf16(bits.astype(np.float64)), want)


def test_round_bf16_ties_subnormals_and_non_finite_values():
    u = 2.0 ** -8                      # half a bfloat16 ulp at 1.0 (8 significand bits: ulp 2^-7)
    cases = {
        1.0: 1.0, -1.0: -1.0, 0.0: 0.0,
        1.0 + u: 1.0,                  # tie, lower neighbour even (mantissa 0)
        1.0 + 3 * u: 1.0 + 4 * u,      # tie, upper neighbour even (mantissa 2)
        -(1.0 + u): -1.0, -(1.0 + 3 * u): -(1.0 + 4 * u),
        1.0 + u + 2.0 ** -23: 1.0 + 2 * u,    # just above the tie: up
        1.0 + u - 2.0 ** -23: 1.0,            # just below: down
        1.0 + 3 * u - 2.0 ** -22: 1.0 + 2 * u,
        2.0 - u: 2.0,                  # tie at the top of a binade carries into the exponent
        3.3895313892515355e38: 3.3895313892515355e38,        # largest finite bfloat16
        3.3965e38: np.inf,             # more than half an ulp (6.6e35) above it: overflows, as the conversion does
        3.3960e38: 3.3895313892515355e38,     # less than half an ulp above it: stays finite
        2.0 ** -126: 2.0 ** -126,      # smallest normal
        2.0 ** -133: 2.0 ** -133,      # smallest bfloat16 subnormal (float32 subnormal with one high bit)
        2.0 ** -134: 0.0,              # half of it: tie to even (zero)
        3 * 2.0 ** -134: 2.0 ** -132,  # 1.5 subnormal ulps: tie, to the even code 2
        2.0 ** -134 + 2.0 ** -149: 2.0 ** -133,
        np.inf: np.inf, -np.inf: -np.inf,
    }
    x = np.array(list(cases.keys()))
    got = orc.round_bf16(x)
    np.testing.assert_array_equal(got, np.array(list(cases.values())))
    # ... and every one of them is what the library conversion gives
    lib = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(got, lib)
    assert np.signbit(orc.round_bf16(np.array([-0.0]))[0])
    assert np.isnan(orc.round_bf16(np.array([np.nan]))[0])
    # idempotent, and the result always has an empty low half
    g = np.random.default_rng(5)
    r = orc.round_bf16(g.standard_normal(10000))
    np.testing.assert_array_equal(orc.round_bf16(r), r)
    assert _is_bf16(r).all()


def test_round_bf16_goes_through_float32():
    """A double that lies just above a bfloat16 tie but rounds onto the tie in float32 is then rounded to even:
    the path computes in float32 and stores bfloat16, so the oracle's storage rounding takes the same two steps."""
    v = 1.0 + 2.0 ** -8 + 2.0 ** -40           # float32(v) == 1 + 2^-8 exactly (the tie)
    assert float(np.float32(v)) == 1.0 + 2.0 ** -8
    assert orc.round_bf16(np.array([v]))[0] == 1.0


# ---------------------------------------------------------------------------
# where the storage mode rounds
# ---------------------------------------------------------------------------

def _one_layer(act=W.ACT_RELU, k=3, c_in=8, c_out=8, hw=6, batch=4):
    t, s = W.Block(), W.Block()
    t.cba(0, c_out, k)
    s.cba(0, c_out, k, act=act)
    return W.Workload("one_layer", batch, (c_in, hw, hw), [t], [s], "bf16", lr=0.05)


def test_storage_mode_rounds_each_stored_tensor_and_nothing_else():
    """One student layer, composed by hand from the plain primitives with a rounding exactly at the
    stores of the bf16 path (input, compute copy of the weights, convolution output, block output, loss
    gradient, gradient of the convolution output): the storage-mode step must give the same numbers, and
    the tensors the path keeps in wider precision (batch statistics, weight / gamma / beta gradients,
    master weights, momentum) must not be rounded."""
    wl = _one_layer()
    o = make_oracle(wl, storage="bf16")
    x = W.make_input(wl)
    acts = o.teacher_relay(x)
    R = orc.round_bf16
    a0 = R(x.astype(np.float64))
    np.testing.assert_array_equal(acts[0].reshape(x.shape), a0)
    # teacher layer: stored weights, inference-mode BN, activation, one rounding at the store
    tw = W.make_param(wl, 0, 0, 0, W.P_WEIGHT, (8, 8, 3, 3))
    tp = [W.make_param(wl, 0, 0, 0, s, (8,)) for s in (W.P_GAMMA, W.P_BETA, W.P_RMEAN, W.P_RVAR)]
    a1 = R(orc.act_fwd(orc.bn_eval(orc.conv_fwd(a0, R(tw), 1, 1), *tp), W.ACT_RELU))
    np.testing.assert_allclose(acts[1].reshape(a1.shape), a1, rtol=0, atol=0)
    # student step by hand
    sw = W.make_param(wl, 1, 0, 0, W.P_WEIGHT, (8, 8, 3, 3)).astype(np.float64)
    gamma, beta = np.ones(8), np.zeros(8)
    loss = o.student_step(1, acts[0], acts[1], wl.lr)
    y = R(orc.conv_fwd(a0, R(sw), 1, 1))
    pre, mean, var = orc.bn_train_fwd(y, gamma, beta)
    out = R(orc.act_fwd(pre, W.ACT_RELU))
    loss_h, ds = orc.mse(out, a1)
    dpre = orc.act_bwd(R(ds), pre, W.ACT_RELU)
    dconv, dg, db = orc.bn_train_bwd(dpre, y, gamma, mean, var)
    dconv = R(dconv)
    dw = orc.conv_wgrad(dconv, a0, 3, 1, 1)
    assert loss == loss_h
    np.testing.assert_array_equal(o.saved(0, 0, o.SAVED_CONV).reshape(y.shape), y)
    np.testing.assert_array_equal(o.saved(0, 0, o.SAVED_MEAN), mean)
    np.testing.assert_array_equal(o.saved(0, 0, o.SAVED_VAR), var)
    np.testing.assert_array_equal(o.value(0, 1).reshape(out.shape), out)
    np.testing.assert_array_equal(o.get_tensor(orc.KIND_GRAD, 1, 0, 0, W.P_WEIGHT, dw.shape), dw)
    np.testing.assert_array_equal(o.get_tensor(orc.KIND_GRAD, 1, 0, 0, W.P_GAMMA, (8,)), dg)
    np.testing.assert_array_equal(o.get_tensor(orc.KIND_GRAD, 1, 0, 0, W.P_BETA, (8,)), db)
    # the update works on the unrounded master weights
    np.testing.assert_array_equal(o.get_tensor(orc.KIND_PARAM, 1, 0, 0, W.P_WEIGHT, dw.shape), sw - wl.lr * dw)
    # stored tensors are bfloat16 codes; statistics, parameter gradients, master weights are not
    assert _is_bf16(o.saved(0, 0, o.SAVED_CONV)).all() and _is_bf16(o.value(0, 1)).all()
    assert _is_bf16(acts[0]).all() and _is_bf16(acts[1]).all()
    for t in (mean, var, dw, dg, db, o.get_tensor(orc.KIND_PARAM, 1, 0, 0, W.P_WEIGHT, dw.shape),
              o.get_tensor(orc.KIND_MOMENTUM, 1, 0, 0, W.P_WEIGHT, dw.shape), o.saved(0, 0, o.SAVED_PRE)):
        assert not _is_bf16(t).all()
    # and the plain mode rounds nothing at all
    p = make_oracle(wl)
    pa = p.teacher_relay(x)
    np.testing.assert_array_equal(pa[0].reshape(x.shape), x.astype(np.float64))
    p.student_step(1, pa[0], pa[1], wl.lr)
    assert not _is_bf16(p.saved(0, 0, p.SAVED_CONV)).all() and not _is_bf16(p.value(0, 1)).all()


def test_storage_mode_rounds_joins_pools_and_accumulated_gradients():
    """Every value of a block with a residual add, a weighted mix and a pool is a bfloat16 code in the
    storage mode (pooling picks stored values, so it needs no rounding of its own)."""
    for wl in (W.Workload("j", 3, (8, 8, 8), *_join_blocks(), "bf16", lr=0.05),):
        o = make_oracle(wl, storage="bf16")
        acts = o.teacher_relay(W.make_input(wl))
        o.student_step(1, acts[0], acts[1], wl.lr)
        for v in range(len(wl.student[0].ops) + 1):
            assert _is_bf16(o.value(0, v)).all(), v


def _join_blocks():
    t, s = W.Block(), W.Block()
    v = t.cba(0, 8, 3); t.pool(v, 2, 2)
    a = s.cba(0, 8, 3, act=W.ACT_NONE)
    b = s.cba(0, 8, 1, act=W.ACT_NONE)
    m = s.mix([a, b], [0.3, 0.7])
    r = s.add(0, m, act=W.ACT_RELU)
    s.pool(r, 2, 2)
    return [t], [s]


# ---------------------------------------------------------------------------
# kink_margin
# ---------------------------------------------------------------------------

def _identity_layer(act, beta, values, c=8):
    """A student block of one 1x1 convolution with the identity as its weight, BN with gamma 1 and the
    given beta, and `act`; the input holds `values` (one row of positions per channel, the same in every
    channel), so the pre-activations are (values - mean) / sqrt(var + eps) + beta in closed form."""
    n = len(values)
    t, s = W.Block(), W.Block()
    t.cba(0, c, 1)
    s.cba(0, c, 1, act=act)
    wl = W.Workload("ident", 1, (c, 1, n), [t], [s], "f32", lr=0.1)
    o = make_oracle(wl)
    o.set_param(1, 0, 0, W.P_WEIGHT, np.eye(c).reshape(c, c, 1, 1))
    o.set_param(1, 0, 0, W.P_BETA, np.full(c, beta))
    x = np.broadcast_to(np.asarray(values, dtype=np.float64), (1, c, 1, n)).copy()
    target = np.zeros(c * n)
    o.student_step(1, x, target, 0.0, orc.MODE_LOSS)
    return o


@pytest.mark.parametrize("h", [1e-3, 1e-6, 2.5e-9])
def test_kink_margin_relu_pre_activation_at_plus_or_minus_h(h):
    """Input +-1 alternating: mean 0, variance 1, x-hat = +-a with a = 1/sqrt(1 + eps).  beta = a + h puts
    the negative half at +h; beta = a - h puts it at -h; either way the margin is h (the other half sits
    at 2a +- h)."""
    a = 1.0 / np.sqrt(1.0 + 1e-5)
    vals = [1.0, -1.0] * 8
    for beta in (a + h, a - h):
        m = _identity_layer(W.ACT_RELU, beta, vals).kink_margin(0)
        assert m == pytest.approx(h, rel=1e-6, abs=1e-15)
    # no activation: no kink at all
    assert _identity_layer(W.ACT_NONE, a + h, vals).kink_margin(0) == np.inf


@pytest.mark.parametrize("h", [1e-3, 1e-7])
def test_kink_margin_relu6_value_at_6_minus_h(h):
    a = 1.0 / np.sqrt(1.0 + 1e-5)
    vals = [1.0, -1.0] * 8
    # upper half at 6 - h, lower half at 6 - h - 2a (far from 0 and 6): the margin is h
    m = _identity_layer(W.ACT_RELU6, 6.0 - h - a, vals).kink_margin(0)
    assert m == pytest.approx(h, rel=1e-6)
    # the same pre-activations under a plain ReLU are ~4 away from its only kink
    m = _identity_layer(W.ACT_RELU, 6.0 - h - a, vals).kink_margin(0)
    assert m == pytest.approx(6.0 - h - 2 * a, rel=1e-9)
    # above 6 counts too
    m = _identity_layer(W.ACT_RELU6, 6.0 + h - a, vals).kink_margin(0)
    assert m == pytest.approx(h, rel=1e-6)


def test_kink_margin_pool_window_gap():
    """A 2x2 / stride-2 pool over a 4x4 image whose four windows have winner-to-runner-up gaps 0.5, g,
    2.0 and (winner <= 0) anything: the margin is g, the smallest gap among windows with a positive
    winner; windows whose winner is not positive pass no gradient after the ReLU and do not count."""
    g = 3e-4
    img = np.array([[5.0, 4.5, 1.0, 1.0 - g],
                    [0.0, 1.0, 0.2, -3.0],
                    [9.0, 7.0, -1.0, -1.0],
                    [1.0, 2.0, -2.0, -1.0 - 1e-9]])
    t, s = W.Block(), W.Block()
    v = t.pool(0, 2, 2); t.cba(v, 8, 1, act=W.ACT_NONE)
    v = s.pool(0, 2, 2); s.cba(v, 8, 1, act=W.ACT_NONE)
    wl = W.Workload("pool", 2, (8, 4, 4), [t], [s], "f32", lr=0.1)
    o = make_oracle(wl)
    x = np.broadcast_to(img, (2, 8, 4, 4)).copy()
    o.student_step(1, x, np.zeros(2 * 8 * 2 * 2), 0.0, orc.MODE_LOSS)
    assert o.kink_margin(0) == pytest.approx(g, rel=1e-9)
    # widening that window's gap moves the margin to the next smallest one (0.5)
    x[:, :, 0, 3] = 0.0
    o.student_step(1, x, np.zeros(2 * 8 * 2 * 2), 0.0, orc.MODE_LOSS)
    assert o.kink_margin(0) == pytest.approx(0.5, rel=1e-12)


def test_kink_margin_takes_the_minimum_over_ops_and_measures_sums_in_units_of_their_rms():
    """A rectified residual sum is not normalised: its distance from the kink is divided by the sum's rms
    (never by less than 1)."""
    t, s = W.Block(), W.Block()
    t.cba(0, 8, 1)
    v = s.cba(0, 8, 1, act=W.ACT_NONE)
    s.add(0, v, act=W.ACT_RELU)
    wl = W.Workload("sum", 1, (8, 1, 16), [t], [s], "f32", lr=0.1)
    o = make_oracle(wl)
    o.set_param(1, 0, 0, W.P_WEIGHT, np.eye(8).reshape(8, 8, 1, 1))
    a = 10.0 / np.sqrt(100.0 + 1e-5)          # x-hat of +-10 (mean 0, variance 100)
    x = np.broadcast_to(np.array([10.0, -10.0] * 8), (1, 8, 1, 16)).copy()
    # sum = x + xhat = +-(10 + a): rms 10 + a, distance from 0 is 10 + a -> margin 1 in rms units
    o.student_step(1, x, np.zeros(8 * 16), 0.0, orc.MODE_LOSS)
    assert o.kink_margin(0) == pytest.approx(1.0, rel=1e-12)
    o.set_param(1, 0, 0, W.P_BETA, np.full(8, 10.0 + a - 0.25))     # lower half of the sums at -0.25
    o.student_step(1, x, np.zeros(8 * 16), 0.0, orc.MODE_LOSS)
    pre = np.array([20.0 + 2 * a - 0.25, -0.25] * 8)
    assert o.kink_margin(0) == pytest.approx(0.25 / np.sqrt(np.mean(pre ** 2)), rel=1e-9)
