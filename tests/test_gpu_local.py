"""bf16 / MFMA path on the REAL graphs of configurations 2-5, every operation of every student block,
elementwise against the plain fp64 oracle primitives at the stated 2e-2 (max-norm relative error per tensor):
convolution outputs, normalised + activated values, pooled / added / mixed values, the loss, the gradient
stored for every value, the gradients of every weight, gamma and beta; batch statistics, running statistics,
momentum and updated parameters to float32 rounding.  See local_parity.py for how each operation is
compared on the tensors the library itself read, which keeps the comparison elementwise at any depth.

Configuration 2 runs at its full batch (256 x 32 x 32); configurations 3-5 at the 224 x 224 image size of
the benchmark with a reduced batch (the direct-loop oracle needs seconds per sample there).  The same walk
at the full batch, restricted to the heaviest layers, is in test_gpu_fullsize.py."""
import numpy as np
import pytest

import local_parity
import parity
from paper_2301_12443_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL_BF16, TOL_F32 = local_parity.TOL_BF16, local_parity.TOL_F32


@pytest.mark.parametrize("name,batch,hw", [("vgg16_dsconv", 256, 32), ("mbv2_mbconv_k5e4", 4, 224),
                                            ("mbv2_supernet", 2, 224), ("resnet50_x1.5", 4, 224)])
def test_every_layer_of_the_real_graphs_against_the_plain_oracle(name, batch, hw):
    wl = W.CONFIGS[name](batch=batch, hw=hw)
    worst = local_parity.run_and_check(wl, batch)
    print(f"[{name}] worst per kind over all blocks: " + ", ".join(f"{k} {v:.1e}" for k, v in sorted(worst.items())), flush=True)


@pytest.mark.parametrize("name", ["l_res_from_input", "l_add_bwd_paths", "l_s2_classes", "l_stem7x7"])
def test_layer_walk_where_adds_losses_and_pools_ride_in_other_kernels(name):
    """Blocks whose residual adds are done inside the batch-norm passes of the layer before them (forward and
    backward), whose loss is formed inside that backward reduction, or whose max-pool normalises what it reads:
    every operation against the plain oracle primitives, as for the real graphs."""
    from helpers import layer_workloads
    wl, batch = [c for c in layer_workloads() if c[0].name == name][0]
    worst = local_parity.run_and_check(wl, batch)
    print(f"[{name}] worst per kind: " + ", ".join(f"{k} {v:.1e}" for k, v in sorted(worst.items())), flush=True)


def test_layer_walk_catches_a_planted_mistake():
    """The walk is only worth something if a wrong tensor fails it: the same check against a reference whose
    parameters are off by a few per cent in one layer (a mistake planted on the oracle's side) must fail."""
    import torch
    wl = W.tiny_cnn()
    d = parity.make_distiller(wl, 8, "bf16")
    d.teacher_relay(torch.from_numpy(W.make_input(wl)).cuda())
    d.student_step(2, wl.lr)
    d.sync()
    par = local_parity.student_params(wl, 1)
    E, T = local_parity.check_block(d, wl, 1, par, wl.lr)
    assert max(E.values()) < TOL_BF16 and max(v for k, v in T.items() if not k.endswith(".undecided")) < TOL_F32
    wrong = dict(par)
    wrong[(1, W.P_WEIGHT)] = par[(1, W.P_WEIGHT)] * (1.0 + 0.05 * np.sign(par[(1, W.P_WEIGHT)]))
    E2, _ = local_parity.check_block(d, wl, 1, wrong, wl.lr)
    assert E2["op1.conv"] > TOL_BF16 and E2["v1.dvalue" if "v1.dvalue" in E2 else "op0.dconv"] > TOL_BF16
    wrong = dict(par)
    wrong[(0, W.P_GAMMA)] = par[(0, W.P_GAMMA)] * 1.05
    E3, _ = local_parity.check_block(d, wl, 1, wrong, wl.lr)
    assert E3["op0.out"] > TOL_BF16 and E3["op0.dconv"] > TOL_BF16
