"""Automatic hybrid distribution (Sec. IV-C): profile every block at the feasible batch sizes, then
search exhaustively for the distribution of blocks and batch shards over N devices whose slowest
device is fastest.

With teacher relaying and decoupled updates (Sec. IV-A, IV-B) the devices form a pipeline whose
throughput is set by the slowest one, so a schedule is scored by its bottleneck.  A schedule cuts
the B blocks into contiguous groups and gives group g a number d_g of devices (sum = N); the d_g
devices of a group each run the group's teacher and student blocks on batch / d_g samples and
share the student gradients (Algorithm 1, share_gradient).  d_g = 1 everywhere is the plain
contiguous distribution; one group with d = N is the paper's internal relaying.

This build has one GPU: the profile is measured here through the library's hot path (the same
kernels at batch, batch/2, batch/3, ...), the schedule and its bottleneck time are a prediction.
The gradient exchange inside a group is modelled as a ring all-reduce over a per-link bandwidth
(default: one xGMI link, 153 GB/s); pass link_gbs=None to leave it out, as the paper's profile does.

    python -m paper_2301_12443_amd.ahd --config resnet50_x1.5 --devices 4
"""
from __future__ import annotations

import argparse
import json
from dataclasses import dataclass, field

import numpy as np

from . import workloads as W


@dataclass
class Profile:
    """times[d][i] = seconds of block i (0-based) at batch // d: teacher forward, student step."""
    batch: int
    splits: tuple
    teacher: dict = field(default_factory=dict)     # d -> np.ndarray [B]
    student: dict = field(default_factory=dict)     # d -> np.ndarray [B]
    grad_bytes: np.ndarray | None = None            # fp32 gradient bytes per student block


@dataclass
class Schedule:
    groups: list            # [(first_block, last_block, devices)], blocks 0-based, inclusive
    group_seconds: list     # per-device step time of each group
    bottleneck: float

    def describe(self) -> str:
        return " | ".join(f"blocks {a + 1}-{b + 1} on {d} device{'s' if d > 1 else ''} (batch/{d}): {t * 1e3:.3f} ms"
                          for (a, b, d), t in zip(self.groups, self.group_seconds))


def compositions(total: int, parts: int):
    """All ways to write `total` as an ordered sum of `parts` positive integers."""
    if parts == 1:
        yield (total,)
        return
    for first in range(1, total - parts + 2):
        for rest in compositions(total - first, parts - 1):
            yield (first,) + rest


def allreduce_seconds(nbytes: float, d: int, link_gbs: float | None) -> float:
    """Ring all-reduce of nbytes over d devices, each step bound by one link."""
    if d <= 1 or not link_gbs:
        return 0.0
    return 2.0 * (d - 1) / d * nbytes / (link_gbs * 1e9)


def group_seconds(prof: Profile, first: int, last: int, d: int, link_gbs: float | None) -> float:
    t = float(prof.teacher[d][first:last + 1].sum() + prof.student[d][first:last + 1].sum())
    if prof.grad_bytes is not None:
        t += allreduce_seconds(float(prof.grad_bytes[first:last + 1].sum()), d, link_gbs)
    return t


def search(prof: Profile, n_devices: int, link_gbs: float | None = 153.0) -> Schedule:
    """Exhaustive search (Sec. IV-C): contiguous block groups x device counts per group."""
    B = len(next(iter(prof.teacher.values())))
    feasible = set(prof.teacher)
    best = None
    for g in range(1, min(B, n_devices) + 1):
        for sizes in compositions(B, g):
            bounds, at = [], 0
            for sz in sizes:
                bounds.append((at, at + sz - 1))
                at += sz
            for devs in compositions(n_devices, g):
                if any(d not in feasible for d in devs):
                    continue
                secs = [group_seconds(prof, a, b, d, link_gbs) for (a, b), d in zip(bounds, devs)]
                worst = max(secs)
                if best is None or worst < best.bottleneck:
                    best = Schedule([(a, b, d) for (a, b), d in zip(bounds, devs)], secs, worst)
    if best is None:
        raise ValueError(f"no schedule: {n_devices} devices over {B} blocks with batch splits {sorted(feasible)}")
    return best


def contiguous_only(prof: Profile, n_devices: int) -> Schedule | None:
    """The naive distribution the paper starts from: whole blocks only, one device per group."""
    B = len(prof.teacher[1])
    if n_devices > B:
        return None
    sub = Profile(prof.batch, (1,), {1: prof.teacher[1]}, {1: prof.student[1]}, prof.grad_bytes)
    best = None
    for sizes in compositions(B, n_devices):
        bounds, at = [], 0
        for sz in sizes:
            bounds.append((at, at + sz - 1))
            at += sz
        secs = [group_seconds(sub, a, b, 1, None) for a, b in bounds]
        if best is None or max(secs) < best.bottleneck:
            best = Schedule([(a, b, 1) for a, b in bounds], secs, max(secs))
    return best


def profile_blocks(wl: W.Workload, splits=(1, 2, 3, 4), steps: int = 20, warmup: int = 3, device="cuda:0") -> Profile:
    """Times every block through the library at batch // d for each feasible d (batch % d == 0):
    teacher block i = pbd_teacher_prefix(i) - pbd_teacher_prefix(i-1), student block i =
    pbd_student_step(i); HIP events on the library's stream, kernels launched directly."""
    import torch
    from . import pbd
    prof = Profile(wl.batch, tuple(d for d in splits if wl.batch % d == 0))
    for d in prof.splits:
        batch = wl.batch // d
        dist = pbd.Distiller(wl, batch=batch)
        dist.bind(device)
        dist.load_params()
        x = torch.from_numpy(W.make_input(wl, batch=batch)).to(device)
        stream = dist._stream

        def timed(fn):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for _ in range(warmup):
                fn()
            dist.sync()
            e0.record(stream)
            for _ in range(steps):
                fn()
            e1.record(stream)
            dist.sync()
            return e0.elapsed_time(e1) * 1e-3 / steps

        prefix = [0.0] + [timed(lambda i=i: dist.teacher_prefix(x, i)) for i in range(1, wl.B + 1)]
        prof.teacher[d] = np.maximum(np.diff(np.array(prefix)), 0.0)
        dist.teacher_relay(x)
        prof.student[d] = np.array([timed(lambda i=i: dist.student_step(i, wl.lr)) for i in range(1, wl.B + 1)])
        del dist
        torch.cuda.empty_cache()
    grad = []
    for b in range(wl.B):
        n = sum(int(np.prod(shape)) for (j, slot), shape in W.param_shapes(wl, W.NET_STUDENT, b).items()
                if slot <= W.P_BETA)
        grad.append(4.0 * n)
    prof.grad_bytes = np.array(grad)
    return prof


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--config", default="vgg16_dsconv", choices=sorted(W.CONFIGS))
    ap.add_argument("--devices", type=int, default=4)
    ap.add_argument("--splits", default="1,2,3,4")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--link-gbs", type=float, default=153.0, help="per-link bandwidth of the gradient all-reduce model; 0 = leave it out")
    args = ap.parse_args()
    wl = W.CONFIGS[args.config]()
    prof = profile_blocks(wl, tuple(int(v) for v in args.splits.split(",")), args.steps)
    best = search(prof, args.devices, args.link_gbs or None)
    naive = contiguous_only(prof, args.devices)
    one = float(prof.teacher[1].sum() + prof.student[1].sum())
    out = {
        "config": wl.name, "batch": wl.batch, "devices": args.devices,
        "profile_ms": {str(d): {"teacher": [round(v * 1e3, 4) for v in prof.teacher[d]],
                                "student": [round(v * 1e3, 4) for v in prof.student[d]]} for d in prof.splits},
        "one_device_ms": round(one * 1e3, 4),
        "contiguous_only": None if naive is None else {"schedule": naive.describe(), "bottleneck_ms": round(naive.bottleneck * 1e3, 4)},
        "ahd": {"schedule": best.describe(), "bottleneck_ms": round(best.bottleneck * 1e3, 4),
                "predicted_speedup_over_one_device": round(one / best.bottleneck, 3)},
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
