"""The layer-by-layer walk of local_parity.py at the FULL batch and image size of configurations 3-5, in the
launch configuration the benchmark times, on the heaviest layers: elementwise against the plain fp64 oracle
primitives at 2e-2.  Covered launch shapes: the 256-row direct-to-LDS implicit GEMM (forward and backward-data)
with batch-norm sums taken from its store and more row tiles than one finalize walks, the stride-2 backward-data
by parity classes, the weight gradient split
768 ways over 802816 pixels, the residual add fused into a normalisation pass and its backward, a backward-data
launch that accumulates onto another reader's gradient, the 256 x 128 tile of a 1.6 M-row pointwise layer, the
5 x 5 and 7 x 7 depthwise tile kernels at 112 x 112, wide 1 x 1 layers over 12544 rows."""
import pytest

import local_parity
from paper_2301_12443_amd import workloads as W

pytestmark = pytest.mark.gpu


def _first(wl, b, pred):
    return next(j for j, op in enumerate(wl.student[b].ops) if pred(op))


def test_resnet50_stage1_and_stage4_layers_at_full_batch():
    wl = W.CONFIGS["resnet50_x1.5"]()
    ops = wl.student[0].ops
    assert (ops[3].k, ops[3].c_out, ops[9].k, ops[9].act, ops[10].type) == (3, 96, 1, W.ACT_NONE, W.OP_ADD)
    assert (wl.student[3].ops[1].k, wl.student[3].ops[1].stride) == (3, 2)
    assert (wl.student[3].ops[11].k, wl.student[3].ops[12].type, len(wl.student[3].ops)) == (1, W.OP_ADD, 13)
    sel = {
        # stage 1 (56 x 56, 802816 rows): 3 x 3 96 -> 96; 1 x 1 96 -> 256 whose output only the fused add reads;
        # value 11 = that add's output, read by a 1 x 1 (backward-data) and by the next add (two gradients meet)
        0: ({3, 9, 10}, {4, 10, 11}),
        # stage 4: the stride-2 3 x 3 768 -> 768 from 14 x 14 (its backward-data takes the input pixels parity class
        # by parity class and writes the gradient of value 1); at 7 x 7 (12544 rows) 3 x 3 768 -> 768 and
        # 1 x 1 768 -> 2048 + fused add; op 11 = the block's last 1 x 1, whose batch-norm backward reduction also does
        # the last add's backward pass and forms the loss and its gradient from S_4 and A_4
        3: ({1, 6, 7, 8, 11}, {1, 7, 8, 12}),
    }
    worst = local_parity.run_and_check(wl, wl.batch, sel)
    print("worst per kind:", {k: f"{v:.1e}" for k, v in sorted(worst.items())}, flush=True)


def test_mobilenet_first_block_at_full_batch():
    """Expand 1 x 1 32 -> 128 over 1605632 rows and the 5 x 5 depthwise at 112 x 112 (configuration 3)."""
    wl = W.CONFIGS["mbv2_mbconv_k5e4"]()
    ops = wl.student[0].ops
    assert (ops[1].k, ops[1].c_out, ops[2].k, ops[2].groups) == (1, 128, 5, 128)
    worst = local_parity.run_and_check(wl, wl.batch, {0: ({1, 2}, {2, 3})})
    print("worst per kind:", {k: f"{v:.1e}" for k, v in sorted(worst.items())}, flush=True)


def test_supernet_7x7_depthwise_candidate_at_full_batch():
    """A 7 x 7 depthwise candidate of the first supernet block at 112 x 112, batch 64 (configuration 4), and the
    weighted sum that mixes the block's six candidates."""
    wl = W.CONFIGS["mbv2_supernet"]()
    j = _first(wl, 0, lambda op: op.type == W.OP_CBA and op.groups > 1 and op.k == 7)
    m = _first(wl, 0, lambda op: op.type == W.OP_MIX)
    worst = local_parity.run_and_check(wl, wl.batch, {0: ({j, m}, {j + 1})})
    print("worst per kind:", {k: f"{v:.1e}" for k, v in sorted(worst.items())}, flush=True)
