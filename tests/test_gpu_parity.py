"""GPU parity: libpbd.so (through the C ABI binding) against the CPU oracle on the same
seeded inputs.

Tolerances (max-norm relative error per tensor, max|a-b| / max|b|):
  * float32 path vs the fp64 oracle: 1e-4 on activations, losses, gradients, momentum,
    updated parameters and running statistics;
  * bf16 path: 2e-2.  Losses and relayed activations are compared with the plain fp64
    oracle.  Gradients are compared with the oracle run with bfloat16 storage rounding, so
    that ReLU masks, pool winners and bf16 codes are decided in the kernel's precision on both
    sides: a gradient summed over a kinked network is discontinuous in those decisions and
    the plain fp64 value is several percent away from ANY bf16-storage evaluation (see
    test_bf16_storage_conditioning in test_oracle_step.py for the oracle-only measurement).
    Where that oracle-vs-oracle deviation of a gradient tensor exceeds 4e-2, the bound for the
    tensor is half of it (see _assert_bf16_step).
"""
import numpy as np
import pytest

import parity
from helpers import layer_workloads, make_oracle, max_rel, pattern_workloads
from paper_2301_12443_amd import pbd, workloads as W

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4
TOL_BF16 = 2e-2


KINK_FLOOR = 2e-6   # float32 runs: a pre-activation closer than this to a kink may fall either side


def _assert_all(errs, tol, keys=None):
    bad = {k: v for k, v in errs.items() if not (v < tol) and (keys is None or any(t in k for t in keys))}
    assert not bad, dict(list(sorted(bad.items(), key=lambda kv: -kv[1]))[:8])


def _assert_bf16_step(errs):
    """Losses, gradients, momentum and updated parameters of a bf16 step against the bf16-storage
    oracle.  Which bf16 code a stored value rounds to is decided by the last float32 bit on the
    GPU and in double by the oracle, so a handful of stored elements differ by one bf16 ulp and the
    gradient moves with them; the size of that sensitivity is what the storage rounding itself does
    to the same tensor (oracle vs oracle, ".noise").  Bound: the larger of 2e-2 and half of it."""
    bad = {}
    for k, v in errs.items():
        if k.endswith(".noise") or ".A" in k:
            continue
        tol = TOL_BF16
        for stem in (".grad", ".mom"):
            if k.endswith(stem):
                tol = max(tol, 0.5 * errs.get(k + ".noise", 0.0))
        if k.endswith(".l2g"):
            tol = max(tol, 0.5 * errs.get(k[:-4] + ".grad.noise", 0.0))
        if not v < tol:
            bad[k] = (v, tol)
    assert not bad, dict(list(sorted(bad.items(), key=lambda kv: -kv[1][0]))[:8])


SMALL = [W.tiny_cnn()] + pattern_workloads()


@pytest.mark.parametrize("wl", SMALL, ids=[w.name for w in SMALL])
def test_f32_path_matches_fp64_oracle(wl):
    """Three consecutive steps (momentum and running statistics in play), every tensor."""
    errs = parity.compare_step(wl, precision="f32", steps=3, kink_floor=KINK_FLOOR)
    _assert_all({k: v for k, v in errs.items() if not k.endswith(".l2g")}, TOL_F32)


@pytest.mark.parametrize("precision", ["f32", "bf16"])
def test_long_columns_take_the_chunked_bn_kernels(precision):
    """Batch 96 gives the first two blocks M = 98304 and 24576 rows: above the whole-column limit (4096 rows
    per channel), so the chunked statistics / finalize / apply kernels run, while the last block (1536 rows)
    stays below it."""
    wl = W.tiny_cnn()
    if precision == "f32":
        errs = parity.compare_step(wl, batch=96, precision="f32", steps=2, kink_floor=KINK_FLOOR)
        _assert_all({k: v for k, v in errs.items() if not k.endswith(".l2g")}, TOL_F32)
    else:
        plain = parity.compare_step(wl, batch=96, precision="bf16", steps=1)
        _assert_all(plain, TOL_BF16, keys=(".A", ".loss"))
        rounded = parity.compare_step(wl, batch=96, precision="bf16", steps=1, storage="bf16", noise=True)
        _assert_bf16_step(rounded)


def test_degenerate_shapes():
    """One block, one 1x1 convolution on a 1x1 image, batch 4 (batch norm over four values per
    channel; at the smallest accepted batch, 2, x-hat is +-1 whatever the input and the weight
    gradient is a pure rounding residue, so there is nothing to compare); and a block of
    stride-2 convolutions on a 3x5 image (every tile ragged)."""
    t, s = W.Block(), W.Block()
    t.cba(0, 8, 1); s.cba(0, 8, 1)
    one = W.Workload("one", 4, (8, 1, 1), [t], [s], "f32", lr=0.1)
    errs = parity.compare_step(one, precision="f32", steps=2, kink_floor=KINK_FLOOR)
    _assert_all({k: v for k, v in errs.items() if not k.endswith(".l2g")}, TOL_F32)
    t, s = W.Block(), W.Block()
    t.cba(0, 24, 3, 2); v = s.cba(0, 8, 3, 2, groups=8); s.cba(v, 24, 1)
    odd = W.Workload("odd", 3, (8, 3, 5), [t], [s], "f32", lr=0.1)
    for precision in ("f32", "bf16"):
        errs = parity.compare_step(odd, precision=precision, steps=1, kink_floor=KINK_FLOOR if precision == "f32" else 0.0,
                                   storage=None if precision == "f32" else "bf16", noise=precision == "bf16")
        if precision == "f32":
            _assert_all({k: v for k, v in errs.items() if not k.endswith(".l2g")}, TOL_F32)
        else:
            _assert_bf16_step(errs)


def test_f32_block_order_is_irrelevant():
    wl = W.tiny_cnn()
    a = parity.compare_step(wl, precision="f32", steps=1, order=(3, 1, 4, 2), kink_floor=KINK_FLOOR)
    _assert_all({k: v for k, v in a.items() if not k.endswith(".l2g")}, TOL_F32)


BF16_CASES = [(W.tiny_cnn(), None)] + [(w, None) for w in pattern_workloads()[:3]] + layer_workloads()


@pytest.mark.parametrize("wl,batch", BF16_CASES, ids=[w.name for w, _ in BF16_CASES])
@pytest.mark.parametrize("direct", [False, True], ids=["mfma", "direct"])
def test_bf16_path_matches_oracle(wl, batch, direct):
    plain = parity.compare_step(wl, batch=batch, precision="bf16", force_direct=direct, steps=1)
    _assert_all(plain, TOL_BF16, keys=(".A", ".loss"))
    rounded = parity.compare_step(wl, batch=batch, precision="bf16", force_direct=direct, steps=1, storage="bf16",
                                  noise=True)
    _assert_bf16_step(rounded)


def _gradient_deviation(wl, batch, get_a, get_b):
    """Per block: median relative L2 deviation of the weight gradients of two evaluations."""
    out = []
    for b in range(wl.B):
        devs = []
        for (j, slot), shape in W.param_shapes(wl, W.NET_STUDENT, b).items():
            if slot == W.P_WEIGHT:
                ga, gb = get_a(b, j, shape), get_b(b, j, shape)
                devs.append(np.linalg.norm(ga - gb) / np.linalg.norm(gb))
        out.append(float(np.median(devs)))
    return out


def _full_config_check(wl, batch):
    """bf16 MFMA path at a configuration's real graph: activations and losses against the plain
    fp64 oracle (losses 2e-2, activations 4e-2) and the bf16-storage oracle (2e-2); weight gradients against the bf16-storage oracle, bounded by the larger of
    2e-2 and 1.5x the deviation the storage rounding itself causes (oracle bf16 vs oracle fp64)."""
    import torch
    d = parity.make_distiller(wl, batch, "bf16")
    o64, o16 = make_oracle(wl, batch), make_oracle(wl, batch, storage="bf16")
    x = W.make_input(wl, batch=batch)
    d.distill_step(torch.from_numpy(x).cuda(), wl.lr)
    d.sync()
    print(f"[{wl.name} N={batch}] gpu step done, oracle fp64 ...", flush=True)
    l64 = o64.relay_step(x, wl.lr)
    print(f"[{wl.name}] oracle bf16-storage ...", flush=True)
    l16 = o16.relay_step(x, wl.lr)
    print(f"[{wl.name}] oracle teacher ...", flush=True)
    acts, acts16 = o64.teacher_relay(x), o16.teacher_relay(x)
    for i in range(wl.B + 1):
        got = d.read_act(i)
        assert max_rel(got, acts16[i]) < TOL_BF16, f"A_{i} vs bf16-storage oracle"
        # plain fp64: half-ulp bf16 storage noise (2^-9 per stored layer) grows like sqrt(depth);
        # the 52-layer MobileNetV2 teacher reaches ~2.5e-2 at its last blocks
        assert max_rel(got, acts[i]) < 2 * TOL_BF16, f"A_{i} vs fp64 oracle"
    lg = d.losses.cpu().numpy()
    assert np.all(np.abs(lg - l64) / l64 < TOL_BF16), (lg, l64)
    gpu = lambda b, j, s: d.read_tensor(pbd.PBD_GRAD, 1, b, j, W.P_WEIGHT, s)
    g64 = lambda b, j, s: o64.get_tensor(1, 1, b, j, W.P_WEIGHT, s)
    g16 = lambda b, j, s: o16.get_tensor(1, 1, b, j, W.P_WEIGHT, s)
    noise = _gradient_deviation(wl, batch, g16, g64)
    dev = _gradient_deviation(wl, batch, gpu, g16)
    print(f"[{wl.name}] gradient deviation gpu-vs-oracle(bf16) {np.round(dev, 4)}; storage noise {np.round(noise, 4)}", flush=True)
    for b in range(wl.B):
        assert dev[b] < max(TOL_BF16, 1.5 * noise[b]), (b, dev, noise)
    return dev, noise


def test_config2_vgg16_full_batch():
    _full_config_check(W.vgg16_dsconv(), 256)


@pytest.mark.parametrize("name,batch,hw", [("mbv2_mbconv_k5e4", 4, 224), ("mbv2_supernet", 2, 160),
                                            ("resnet50_x1.5", 2, 160)])
def test_configs_3_to_5_reduced_batch_bf16(name, batch, hw):
    """Same graphs as the full configurations, smaller batch (and image) so that the direct-loop
    oracle finishes; BN statistics depend on the batch, so both sides use the reduced one."""
    _full_config_check(W.CONFIGS[name](batch=batch, hw=hw), batch)


@pytest.mark.parametrize("name,batch,hw,shift", [("vgg16_dsconv", 4, 32, 6.0), ("mbv2_mbconv_k5e4", 4, 96, 3.0),
                                                  ("mbv2_supernet", 2, 64, 3.0), ("resnet50_x1.5", 4, 64, 6.0)])
def test_configs_2_to_5_graphs_in_f32(name, batch, hw, shift):
    """Every op of every block of the real graphs, float32 kernels against the fp64 oracle: pins the
    executor (joins, gradient accumulation, skipped backward-data, update) on the full DAGs.

    A block of these graphs holds ~10^6 rectified elements, so at the default beta = 0 some element
    always sits within float32 rounding of a ReLU kink, where the gradient has two valid values and
    one flip moves every gradient upstream by percents.  The student's beta is therefore set to
    `shift` on both sides (pre-activations ~ N(shift, 1), inside the linear part of ReLU / ReLU6),
    which keeps the comparison elementwise; the kinks themselves are covered at beta = 0 by the
    small workloads above, whose inputs are drawn clear of every kink.  Max-pool ties are not moved
    by beta (two window elements within rounding of each other send the gradient to either
    position), so each block's input is also redrawn until the oracle sees no such near-tie: at
    |value| ~ 10 a float32 activation carries a few 1e-6 of rounding, hence the 1e-5 floor."""
    wl = W.CONFIGS[name](batch=batch, hw=hw, precision="f32")
    errs = parity.compare_step(wl, batch=batch, precision="f32", steps=1, beta_shift=shift, kink_floor=1e-5)
    # the last blocks normalise over as few as 16 samples per channel at these batch sizes and
    # BN backward amplifies float32 rounding accordingly: 5e-4 here, 1e-4 on the tiny config above
    _assert_all({k: v for k, v in errs.items() if not k.endswith(".l2g")}, 5 * TOL_F32)
