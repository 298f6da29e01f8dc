"""Pins for the oracle's architecture round (Sec. VI-A, neural architecture search: a second
forward/backward round per step trains the architecture parameters with the weights frozen)."""
import numpy as np
import pytest
import torch

import torch_ref
from helpers import make_oracle, max_rel, mix_ops, skip_mix, supernet, twin_candidates
from oracle import pbd_oracle as orc
from paper_2301_12443_amd import workloads as W


def test_alpha_gradient_matches_finite_differences():
    """Central differences of loss_i over every architecture parameter."""
    for wl in (supernet(), twin_candidates(4, W.ACT_RELU), skip_mix()):
        o = make_oracle(wl)
        rng = np.random.default_rng(3)
        acts = o.teacher_relay(W.make_input(wl))
        alphas = {j: rng.normal(0.0, 0.7, n) for j, n in mix_ops(wl)}
        for j, a in alphas.items():
            o.set_alpha(0, j, a)
        o.student_step(1, acts[0], acts[1], 0.0, orc.MODE_ARCH_GRADS)
        for j, a in alphas.items():
            g = o.get_alpha(0, j, a.size, orc.ALPHA_GRAD)
            assert a.size == 1 or np.max(np.abs(g)) > 1e-6      # the check below is not vacuous
            for k in range(a.size):
                errs = []
                for h in (1e-5, 1e-6, 1e-7):
                    e = np.zeros_like(a); e[k] = h
                    o.set_alpha(0, j, a + e)
                    lp = o.student_step(1, acts[0], acts[1], 0.0, orc.MODE_LOSS)
                    o.set_alpha(0, j, a - e)
                    lm = o.student_step(1, acts[0], acts[1], 0.0, orc.MODE_LOSS)
                    errs.append(abs((lp - lm) / (2 * h) - g[k]))
                o.set_alpha(0, j, a)
                assert min(errs) <= 1e-6 * np.max(np.abs(g)) + 1e-10, (wl.name, j, k, g[k], errs)


def test_two_round_step_matches_pytorch_autograd():
    """Three NAS steps, each an architecture round then a weight round on the same batch: alpha with
    its gradient and momentum, the weights the first round must not touch, losses, running statistics."""
    wl = supernet()
    o = make_oracle(wl)
    lr_alpha = 0.3
    tpar = torch_ref.block_params(wl, W.NET_TEACHER, 0, False)
    spar = torch_ref.block_params(wl, W.NET_STUDENT, 0, True)
    wkeys = [k for k, v in spar.items() if v.requires_grad]
    wmom = {k: torch.zeros_like(spar[k]) for k in wkeys}
    alphas = {j: torch.log(torch.tensor(wl.student[0].ops[j].p, dtype=torch.float64)).requires_grad_()
              for j, _ in mix_ops(wl)}
    amom = {j: torch.zeros_like(a) for j, a in alphas.items()}
    shapes = W.activation_shapes(wl)

    def running_stats(stats):
        with torch.no_grad():
            for j, (mu, var) in stats.items():
                cnt = wl.batch * np.prod(W.block_shapes(wl.student[0], shapes[0])[j + 1][1:])
                spar[(j, W.P_RMEAN)].mul_(0.9).add_(0.1 * mu)
                spar[(j, W.P_RVAR)].mul_(0.9).add_(0.1 * var * cnt / (cnt - 1))

    for step in range(3):
        x = W.make_input(wl, step=step)
        acts = o.teacher_relay(x)
        a_prev = torch.from_numpy(x).double()
        with torch.no_grad():
            a_i, _ = torch_ref.run_block(wl.teacher[0], a_prev, tpar, train=False)
        # ---- architecture round ----
        before = {k: o.get_tensor(orc.KIND_PARAM, 1, 0, k[0], k[1], spar[k].shape).copy() for k in wkeys}
        loss_o = o.student_step(1, acts[0], acts[1], lr_alpha, orc.MODE_ARCH_STEP)
        out, stats = torch_ref.run_block(wl.student[0], a_prev, spar, train=True, alphas=alphas)
        loss_t = torch.mean((out - a_i) ** 2)
        assert abs(loss_o - loss_t.item()) <= 1e-11 * abs(loss_t.item())
        grads = torch.autograd.grad(loss_t, list(alphas.values()))
        running_stats(stats)
        with torch.no_grad():
            for (j, a), g in zip(alphas.items(), grads):
                assert max_rel(o.get_alpha(0, j, a.numel(), orc.ALPHA_GRAD), g.numpy()) < 1e-9, (step, j)
                amom[j].mul_(wl.momentum).add_(g)
                a.sub_(lr_alpha * amom[j])
                assert max_rel(o.get_alpha(0, j, a.numel(), orc.ALPHA_MOMENTUM), amom[j].numpy()) < 1e-9
                assert max_rel(o.get_alpha(0, j, a.numel()), a.numpy()) < 1e-10
                assert max_rel(o.get_alpha(0, j, a.numel(), orc.ALPHA_PROB), torch.softmax(a, 0).numpy()) < 1e-12
        for k in wkeys:      # frozen in this round, bit for bit
            assert np.array_equal(before[k], o.get_tensor(orc.KIND_PARAM, 1, 0, k[0], k[1], spar[k].shape))
        for j in stats:
            np.testing.assert_allclose(o.get_tensor(0, 1, 0, j, W.P_RMEAN, spar[(j, W.P_RMEAN)].shape),
                                       spar[(j, W.P_RMEAN)].numpy(), rtol=1e-10, atol=1e-14)
        # ---- weight round, mixing with the alpha just trained ----
        loss_o = o.student_step(1, acts[0], acts[1], wl.lr, orc.MODE_STEP)
        out, stats = torch_ref.run_block(wl.student[0], a_prev, spar, train=True, alphas=alphas)
        loss_t = torch.mean((out - a_i) ** 2)
        assert abs(loss_o - loss_t.item()) <= 1e-11 * abs(loss_t.item())
        grads = torch.autograd.grad(loss_t, [spar[k] for k in wkeys])
        running_stats(stats)
        with torch.no_grad():
            for k, g in zip(wkeys, grads):
                assert max_rel(o.get_tensor(orc.KIND_GRAD, 1, 0, k[0], k[1], g.shape), g.numpy()) < 1e-9
                wmom[k].mul_(wl.momentum).add_(g)
                spar[k].sub_(wl.lr * wmom[k])
                assert max_rel(o.get_tensor(orc.KIND_PARAM, 1, 0, k[0], k[1], g.shape), spar[k].numpy()) < 1e-10
        for j, a in alphas.items():   # and the weight round leaves alpha alone
            assert max_rel(o.get_alpha(0, j, a.numel()), a.detach().numpy()) < 1e-10


def test_alpha_gradient_sums_to_zero_and_vanishes_for_identical_candidates():
    """softmax is invariant under a common shift of alpha, so the gradient has no component along
    (1,...,1); candidates that compute the same function cannot be told apart, so it vanishes."""
    wl = twin_candidates(3)
    o = make_oracle(wl)
    acts = o.teacher_relay(W.make_input(wl))
    (j, n), = mix_ops(wl)
    o.set_alpha(0, j, [0.3, -1.0, 0.5])
    o.student_step(1, acts[0], acts[1], 0.0, orc.MODE_ARCH_GRADS)
    g = o.get_alpha(0, j, n, orc.ALPHA_GRAD)
    assert np.max(np.abs(g)) > 1e-4
    assert abs(g.sum()) < 1e-14 * np.max(np.abs(g)) * 100
    # copy candidate 0's parameters into the others
    shapes = W.param_shapes(wl, W.NET_STUDENT, 0)
    for (jj, slot), shape in shapes.items():
        if jj in (0, 1):
            src = o.get_tensor(orc.KIND_PARAM, 1, 0, jj, slot, shape)
            for twin in (jj + 2, jj + 4):
                o.set_param(1, 0, twin, slot, src)
    o.student_step(1, acts[0], acts[1], 0.0, orc.MODE_ARCH_GRADS)
    g2 = o.get_alpha(0, j, n, orc.ALPHA_GRAD)
    assert np.max(np.abs(g2)) < 1e-12 * np.max(np.abs(g))


def test_alpha_starts_at_the_log_of_the_descriptor_weights():
    wl = supernet()
    o = make_oracle(wl)
    acts = o.teacher_relay(W.make_input(wl))
    loss_p = o.student_step(1, acts[0], acts[1], 0.0, orc.MODE_LOSS)
    with pytest.raises(ValueError):
        o.get_alpha(0, mix_ops(wl)[0][0], 3)                     # not defined before the first round
    loss_a = o.student_step(1, acts[0], acts[1], 0.0, orc.MODE_ARCH_GRADS)
    assert abs(loss_a - loss_p) <= 1e-14 * loss_p
    for j, n in mix_ops(wl):
        p = np.array(wl.student[0].ops[j].p)
        np.testing.assert_allclose(o.get_alpha(0, j, n), np.log(p), rtol=1e-15)
        np.testing.assert_allclose(o.get_alpha(0, j, n, orc.ALPHA_PROB), p, rtol=1e-15)
    with pytest.raises(ValueError):
        o.set_alpha(0, 0, [0.0, 0.0, 0.0])                       # op 0 is a convolution
    with pytest.raises(ValueError):
        o.set_alpha(0, mix_ops(wl)[0][0], [0.0, 0.0])            # wrong count


def test_relay_arch_step_is_the_per_block_round():
    wl = supernet()
    a, b = make_oracle(wl), make_oracle(wl)
    x = W.make_input(wl)
    la = a.relay_arch_step(x, 0.2)
    acts = b.teacher_relay(x)
    lb = [b.student_step(i + 1, acts[i], acts[i + 1], 0.2, orc.MODE_ARCH_STEP) for i in range(wl.B)]
    assert np.array_equal(la, np.array(lb))
    for j, n in mix_ops(wl):
        assert np.array_equal(a.get_alpha(0, j, n), b.get_alpha(0, j, n))


def test_mix_alpha_grad_primitive_against_autograd():
    """The exported primitive on its own: dL/dalpha of z = sum_k softmax(alpha)_k y_k for a linear loss <c, z>
    against PyTorch autograd with alpha as a leaf, and its two invariants (components sum to zero; identical
    candidates give zero)."""
    import torch
    g = np.random.default_rng(3)
    n, numel = 5, 257
    ys = g.standard_normal((n, numel))
    c = g.standard_normal(numel)
    alpha = torch.tensor(g.standard_normal(n), dtype=torch.float64, requires_grad=True)
    p = torch.softmax(alpha, 0)
    loss = torch.dot(torch.from_numpy(c), (p[:, None] * torch.from_numpy(ys)).sum(0))
    (ref,) = torch.autograd.grad(loss, alpha)
    got = orc.mix_alpha_grad(c, list(ys), p.detach().numpy())
    np.testing.assert_allclose(got, ref.numpy(), rtol=1e-12, atol=1e-14)
    assert abs(got.sum()) < 1e-12 * np.abs(got).max()
    same = orc.mix_alpha_grad(c, [ys[0]] * n, p.detach().numpy())
    assert np.abs(same).max() < 1e-12 * abs(np.dot(c, ys[0]))
