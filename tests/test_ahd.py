"""Automatic hybrid distribution (Sec. IV-C): the brute-force oracle against hand-worked cases and a
pipeline simulation, and the library's search against the oracle."""
from math import comb

import numpy as np
import pytest

from oracle import ahd_oracle as O
from paper_2301_12443_amd import ahd


def _tables(rng, n_blocks, splits, overhead=0.15):
    """Random per-block times whose batch scaling is imperfect: t(batch/d) = t(batch)/d + a fixed part."""
    base_t = rng.uniform(0.2, 2.0, n_blocks)
    base_s = rng.uniform(0.5, 6.0, n_blocks)
    fixed = rng.uniform(0.0, overhead, n_blocks)
    tt = {d: base_t / d + (fixed if d > 1 else 0) for d in splits}
    ts = {d: base_s / d + (2 * fixed if d > 1 else 0) for d in splits}
    return tt, ts


def _profile(tt, ts, grad_bytes=None):
    return ahd.Profile(256, tuple(sorted(tt)), {d: np.asarray(v) for d, v in tt.items()},
                       {d: np.asarray(v) for d, v in ts.items()},
                       None if grad_bytes is None else np.asarray(grad_bytes, dtype=np.float64))


# ---- the oracle against cases worked by hand -----------------------------------------------------------

def test_oracle_hand_worked_heavy_first_block():
    """Two blocks, three devices.  Block 1 is heavy and scales imperfectly:
         batch/1: (3.0, 1.0)   batch/2: (1.6, 0.6)   batch/3: (1.3, 0.5)        (teacher+student per block)
       {1,1 | 2}: max(1.6, 1.0) = 1.6     {1 | 2,2}: max(3.0, 0.6) = 3.0     {12,12,12}: 1.3+0.5 = 1.8
       so the hybrid split of block 1 over two devices wins with 1.6 (the case of Fig. 3c)."""
    tt = {1: [1.0, 0.25], 2: [0.5, 0.1], 3: [0.4, 0.1]}
    ts = {1: [2.0, 0.75], 2: [1.1, 0.5], 3: [0.9, 0.4]}
    best, intervals = O.brute_force(tt, ts, 3)
    assert best == pytest.approx(1.6)
    assert intervals == ((0, 0), (0, 0), (1, 1))
    # with perfect scaling the whole batch split three ways is best: (3 + 1) / 3
    tt = {d: [1.0 / d, 0.25 / d] for d in (1, 2, 3)}
    ts = {d: [2.0 / d, 0.75 / d] for d in (1, 2, 3)}
    best, intervals = O.brute_force(tt, ts, 3)
    assert best == pytest.approx(4.0 / 3.0)
    assert intervals == ((0, 1),) * 3


def test_oracle_equal_blocks_one_each():
    """B equal blocks on B devices whose times do not shrink with the batch: one block per device."""
    tt = {d: [0.5] * 4 for d in (1, 2, 3, 4)}
    ts = {d: [1.5] * 4 for d in (1, 2, 3, 4)}
    best, intervals = O.brute_force(tt, ts, 4)
    assert best == pytest.approx(2.0)
    assert intervals == ((0, 0), (1, 1), (2, 2), (3, 3))


def test_oracle_counts_every_valid_distribution():
    """With splits up to N all allowed, the valid distributions of B blocks over N devices are the pairs
    (composition of B into g parts, composition of N into g parts): sum_g C(B-1,g-1) C(N-1,g-1)."""
    import itertools
    for n_blocks, n_dev in ((3, 2), (4, 3), (4, 4), (2, 4)):
        ivs = [(a, b) for a in range(n_blocks) for b in range(a, n_blocks)]
        count = sum(O.is_valid(c, n_blocks) for c in itertools.product(ivs, repeat=n_dev))
        want = sum(comb(n_blocks - 1, g - 1) * comb(n_dev - 1, g - 1) for g in range(1, min(n_blocks, n_dev) + 1))
        assert count == want


def test_oracle_unprofiled_split_is_not_used():
    tt = {1: [1.0, 1.0], 2: [0.5, 0.5]}
    ts = {1: [1.0, 1.0], 2: [0.5, 0.5]}
    best, intervals = O.brute_force(tt, ts, 3)        # 3-way split was never profiled
    assert intervals in (((0, 0), (0, 0), (1, 1)), ((0, 0), (1, 1), (1, 1)))
    assert best == pytest.approx(2.0)


def test_simulated_pipeline_runs_at_the_bottleneck():
    """Steady state of the relayed pipeline with decoupled updates: one step per bottleneck time
    (Sec. IV-B); the makespan of K steps lies between K x bottleneck and that plus one pipeline fill."""
    rng = np.random.default_rng(5)
    for _ in range(20):
        n_blocks = int(rng.integers(2, 6))
        tt, ts = _tables(rng, n_blocks, (1, 2, 3, 4))
        cut = int(rng.integers(1, n_blocks))
        groups = [(0, cut - 1, int(rng.integers(1, 4))), (cut, n_blocks - 1, int(rng.integers(1, 4)))]
        per_group = [O.device_seconds(tt, ts, a, b, d) for a, b, d in groups]
        k = 200
        span = O.simulate(groups, tt, ts, k)
        assert span >= k * max(per_group) - 1e-9
        assert span <= k * max(per_group) + sum(per_group) + 1e-9
        assert O.simulate(groups, tt, ts, 2 * k) - span == pytest.approx(k * max(per_group), rel=1e-9)


def test_simulation_of_one_step_is_the_critical_path():
    """One step, two groups, worked by hand: group 2 waits for group 1's teacher only."""
    tt = {1: [1.0, 2.0]}
    ts = {1: [5.0, 3.0]}
    assert O.simulate([(0, 0, 1), (1, 1, 1)], tt, ts, 1) == pytest.approx(max(1.0 + 5.0, 1.0 + 2.0 + 3.0))
    assert O.simulate([(0, 1, 1)], tt, ts, 1) == pytest.approx(11.0)


# ---- the library's search against the oracle -----------------------------------------------------------

def test_compositions():
    for total in range(1, 8):
        for parts in range(1, total + 1):
            got = list(ahd.compositions(total, parts))
            assert len(got) == comb(total - 1, parts - 1) == len(set(got))
            assert all(sum(c) == total and min(c) >= 1 for c in got)


@pytest.mark.parametrize("splits", [(1, 2, 3, 4), (1, 2), (1, 2, 4)])
def test_search_matches_brute_force(splits):
    rng = np.random.default_rng(len(splits))
    for trial in range(12):
        n_blocks = int(rng.integers(2, 6))
        n_dev = int(rng.integers(1, 5))
        tt, ts = _tables(rng, n_blocks, splits, overhead=float(rng.uniform(0.0, 0.8)))
        want, intervals = O.brute_force(tt, ts, n_dev)
        got = ahd.search(_profile(tt, ts), n_dev, link_gbs=None)
        assert got.bottleneck == pytest.approx(want, rel=1e-12)
        # the schedule is a valid distribution with that score
        assert sum(d for _, _, d in got.groups) == n_dev
        assert got.groups[0][0] == 0 and got.groups[-1][1] == n_blocks - 1
        assert all(b[0] == a[1] + 1 for a, b in zip(got.groups, got.groups[1:]))
        per_dev = tuple((a, b) for a, b, d in got.groups for _ in range(d))
        assert O.is_valid(per_dev, n_blocks)
        assert max(O.device_seconds(tt, ts, a, b, d) for a, b, d in got.groups) == pytest.approx(want)
        # and the simulated pipeline runs at that rate
        k = 100
        grown = O.simulate(got.groups, tt, ts, 2 * k) - O.simulate(got.groups, tt, ts, k)
        assert grown == pytest.approx(k * want, rel=1e-9)


def test_search_with_the_gradient_exchange():
    """A ring all-reduce moves 2 (d-1)/d of the bytes through each link."""
    assert ahd.allreduce_seconds(1e9, 1, 100.0) == 0.0
    assert ahd.allreduce_seconds(1e9, 2, 100.0) == pytest.approx(0.01)
    assert ahd.allreduce_seconds(1e9, 4, 100.0) == pytest.approx(0.015)
    assert ahd.allreduce_seconds(1e9, 4, None) == 0.0
    rng = np.random.default_rng(11)
    for trial in range(8):
        n_blocks, n_dev = int(rng.integers(2, 5)), int(rng.integers(2, 5))
        tt, ts = _tables(rng, n_blocks, (1, 2, 3, 4))
        nbytes = rng.uniform(1e7, 4e8, n_blocks)
        link = 1.0      # GB/s: slow enough for the exchange to change the answer

        def comm(first, last, d):
            sent = 0.0
            for step in range(2 * (d - 1)):                 # reduce-scatter, then all-gather
                sent += nbytes[first:last + 1].sum() / d    # one chunk per step per link
            return sent / (link * 1e9)

        want, _ = O.brute_force(tt, ts, n_dev, comm)
        got = ahd.search(_profile(tt, ts, nbytes), n_dev, link_gbs=link)
        assert got.bottleneck == pytest.approx(want, rel=1e-12)
        free, _ = O.brute_force(tt, ts, n_dev)
        assert want >= free


def test_contiguous_only_is_the_all_ones_case():
    rng = np.random.default_rng(3)
    tt, ts = _tables(rng, 5, (1, 2, 3, 4))
    want, _ = O.brute_force({1: tt[1]}, {1: ts[1]}, 3)
    got = ahd.contiguous_only(_profile(tt, ts), 3)
    assert got.bottleneck == pytest.approx(want)
    assert all(d == 1 for _, _, d in got.groups)
    assert ahd.contiguous_only(_profile(tt, ts), 6) is None      # more devices than blocks
    assert ahd.search(_profile(tt, ts), 3, None).bottleneck <= got.bottleneck


def test_search_rejects_an_impossible_request():
    tt, ts = {1: np.ones(2)}, {1: np.ones(2)}
    with pytest.raises(ValueError):
        ahd.search(_profile(tt, ts), 3, None)       # 3 devices, 2 blocks, no batch split profiled


@pytest.mark.gpu
def test_profile_through_the_library_and_schedule():
    """The profile is taken through the C ABI at batch and batch/2; its times are positive and the
    schedule found for it covers every block."""
    from paper_2301_12443_amd import workloads as W
    wl = W.tiny_cnn(batch=16)
    prof = ahd.profile_blocks(wl, splits=(1, 2, 3), steps=5, warmup=2)
    assert prof.splits == (1, 2)                                 # 16 % 3 != 0
    for d in prof.splits:
        assert prof.teacher[d].shape == prof.student[d].shape == (wl.B,)
        assert np.all(prof.teacher[d] >= 0) and np.all(prof.student[d] > 0)
        assert np.all(prof.student[d] < 1.0)                     # seconds
    assert prof.grad_bytes.shape == (wl.B,) and np.all(prof.grad_bytes > 0)
    best = ahd.search(prof, 4)
    assert sum(d for _, _, d in best.groups) == 4
    assert best.groups[0][0] == 0 and best.groups[-1][1] == wl.B - 1
    tt = {d: list(v) for d, v in prof.teacher.items()}
    ts = {d: list(v) for d, v in prof.student.items()}
    want, _ = O.brute_force(tt, ts, 4, lambda a, b, d: ahd.allreduce_seconds(prof.grad_bytes[a:b + 1].sum(), d, 153.0))
    assert best.bottleneck == pytest.approx(want, rel=1e-12)
