"""Host logic of the benchmark's report: which kernel class is reported, against which roofline."""
import pytest

import bench


def _entry(name, ms, nbytes, flops=0.0):
    return dict(name=name, ms=ms, bytes=nbytes, flops=flops, net=1, block=0, op=0)


def test_bandwidth_bound_class_is_reported_against_hbm():
    steps = 2
    prof = []
    for _ in range(steps):
        prof += [_entry("bn_bwd_reduce", 0.020, 40e6)] * 3          # 60 us per step: the most time
        prof += [_entry("igemm_fwd_128x128_store", 0.050, 10e6, 2e10)]
    roof, classes, totals = bench.roofline_from_profile(prof, steps)
    assert roof["kernel"] == "bn_bwd_reduce" and roof["bound"] == "hbm" and roof["unit"] == "GB/s"
    assert roof["launches_per_step"] == roof["class_launches_per_step"] == 3
    assert roof["avg_launch_us"] == pytest.approx(20.0)
    assert roof["achieved"] == pytest.approx(40e6 / 20e-6 / 1e9)     # bytes of one launch over its duration
    assert roof["frac"] == pytest.approx(roof["achieved"] / bench.PEAK_HBM_GBS, abs=1e-4)
    assert classes["bn_bwd_reduce"]["ms_per_step"] == pytest.approx(0.060)
    assert totals["launches"] == 4
    assert totals["algorithmic_bytes"] == pytest.approx(3 * 40e6 + 10e6)
    assert totals["algorithmic_flops"] == pytest.approx(2e10)
    assert totals["kernel_ms"] == pytest.approx(0.110)


def test_contraction_counts_against_mfma_only_above_the_ridge():
    ridge = bench.PEAK_BF16_TFLOPS * 1e12 / (bench.PEAK_HBM_GBS * 1e9)          # flop per byte
    hi = _entry("wgrad_128x128", 0.200, 100e6, 100e6 * ridge * 4)               # 3x3 layer: well above
    lo = _entry("wgrad_128x128", 0.100, 400e6, 400e6 * ridge / 4)               # 1x1 layer: below
    roof, _, _ = bench.roofline_from_profile([hi, hi, lo], 1)
    assert roof["kernel"] == "wgrad_128x128" and roof["bound"] == "mfma" and roof["unit"] == "TFLOP/s"
    assert (roof["launches_per_step"], roof["class_launches_per_step"]) == (2, 3)
    assert roof["achieved"] == pytest.approx(hi["flops"] / 200e-6 / 1e12, rel=1e-3)
    assert roof["peak"] == bench.PEAK_BF16_TFLOPS
    # the same class with most of its time below the ridge is a bandwidth figure
    roof, _, _ = bench.roofline_from_profile([hi, lo, lo, lo], 1)
    assert roof["bound"] == "hbm" and roof["launches_per_step"] == 3
    assert roof["achieved"] == pytest.approx(400e6 / 100e-6 / 1e9)


def test_depthwise_counts_against_the_vector_alu_peak():
    ridge = bench.PEAK_FP32_VALU_TFLOPS * 1e12 / (bench.PEAK_HBM_GBS * 1e9)
    k7 = _entry("dw_fwd_tile_k7", 0.070, 100e6, 100e6 * ridge * 2.5)
    k3 = _entry("dw_fwd_tile_k3", 0.030, 100e6, 100e6 * ridge * 0.4)
    roof, _, _ = bench.roofline_from_profile([k7, k3], 1)
    assert roof["kernel"] == "dw_fwd_tile_k7" and roof["bound"] == "alu" and roof["peak"] == bench.PEAK_FP32_VALU_TFLOPS
    roof, _, _ = bench.roofline_from_profile([k3], 1)
    assert roof["bound"] == "hbm"


def test_more_than_one_gpu_is_refused(monkeypatch, capsys):
    monkeypatch.setattr("sys.argv", ["bench.py", "--gpus", "2"])
    with pytest.raises(SystemExit) as e:
        bench.main()
    assert e.value.code == 2
    assert "single-GPU" in capsys.readouterr().err


def test_capture_order_tuning_keeps_the_fastest_permutation():
    """The tuner tries permutations of the B+1 branches only, always from an empty pipeline, and leaves
    the fastest one set."""
    import time
    from types import SimpleNamespace

    class FakeDistiller:
        def __init__(self, slow_unless):
            self.order, self.pending, self.tried, self.fast = None, False, [], slow_unless

        def set_pipeline_order(self, order):
            assert not self.pending
            self.order = list(order)
            self.tried.append(self.order)

        def pipeline_step(self, x, lr):
            self.pending = True
            if self.order != self.fast:
                time.sleep(0.0005)

        def pipeline_flush(self):
            self.pending = False

    wl = SimpleNamespace(B=4, lr=0.1)
    torch = SimpleNamespace(cuda=SimpleNamespace(synchronize=lambda: None))
    d = FakeDistiller(slow_unless=[1, 0, 2, 3, 4])
    best = bench.tune_pipeline_order(d, None, wl, torch, tries=10)
    assert best == [1, 0, 2, 3, 4] == d.order and not d.pending
    assert d.tried[0] == [0, 1, 2, 3, 4]                       # the default is among the candidates
    assert all(sorted(o) == [0, 1, 2, 3, 4] for o in d.tried)
    assert len({tuple(o) for o in d.tried[:-1]}) == len(d.tried) - 1 == wl.B + 3


def test_family_fractions_split_convolutions_at_the_ridge():
    """The metric's second half: convolutions against the MFMA peak (all launches, and those above / below
    the ridge), bandwidth-bound families against the HBM peak; time-weighted, per step."""
    ridge = bench.PEAK_BF16_TFLOPS * 1e12 / (bench.PEAK_HBM_GBS * 1e9)
    hi = _entry("igemm_fwd_128x128_store", 0.200, 100e6, 100e6 * ridge * 4)
    lo = _entry("wgrad_128x128", 0.100, 400e6, 400e6 * ridge / 4)
    bn = _entry("bn_apply", 0.050, 300e6)
    dw = _entry("dw_fwd_tile_k5", 0.150, 500e6, 1e9)
    other = _entry("unknown_kernel", 1.0, 1e6)
    conv, ew = bench.family_fractions([hi, lo, bn, dw, other] * 2, 2)
    assert conv["launches_per_step"] == 2 and conv["ms_per_step"] == pytest.approx(0.300)
    assert conv["TFLOPs"] == pytest.approx((hi["flops"] + lo["flops"]) / 300e-6 / 1e12, rel=1e-3)
    assert conv["frac_of_mfma_peak"] == pytest.approx(conv["TFLOPs"] / bench.PEAK_BF16_TFLOPS, abs=1e-4)
    assert conv["above_ridge"]["launches_per_step"] == 1
    assert conv["above_ridge"]["TFLOPs"] == pytest.approx(hi["flops"] / 200e-6 / 1e12, rel=1e-3)
    assert conv["below_ridge"]["GBs"] == pytest.approx(400e6 / 100e-6 / 1e9, rel=1e-3)
    assert ew["launches_per_step"] == 2 and ew["ms_per_step"] == pytest.approx(0.200)
    assert ew["GBs"] == pytest.approx(800e6 / 200e-6 / 1e9, rel=1e-3)
    assert ew["frac_of_hbm_peak"] == pytest.approx(ew["GBs"] / bench.PEAK_HBM_GBS, abs=1e-4)
