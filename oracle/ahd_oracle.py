"""Brute-force oracle for automatic hybrid distribution (Sec. IV-C) and a step-by-step simulation of
the relayed pipeline it schedules (Sec. IV-A, IV-B, Algorithm 1).

TEST INFRASTRUCTURE ONLY: imported by tests/, never by the product package, and it imports nothing
from there.  Pure Python loops over tiny cases.

A distribution gives every device one interval of blocks.  It is valid when, walking the devices in
rank order, each interval either repeats the previous one (those devices form a group that splits the
batch evenly and shares gradients) or starts at the block after the previous interval ends; the first
interval starts at block 0 and the last ends at block B-1, so every block runs somewhere and the relay
only ever goes to the next rank.  A group of d devices must have a profiled time at batch / d.
The score of a distribution is the step time of its slowest device.
"""
from __future__ import annotations

import itertools


def device_seconds(t_teacher, t_student, first, last, d, comm=None):
    """One device of a d-wide group owning blocks first..last: its teacher blocks, then its student
    blocks, at batch / d; comm(first, last, d) adds the gradient exchange when given."""
    t = 0.0
    for i in range(first, last + 1):
        t += t_teacher[d][i] + t_student[d][i]
    if comm is not None:
        t += comm(first, last, d)
    return t


def is_valid(intervals, n_blocks):
    if intervals[0][0] != 0 or intervals[-1][1] != n_blocks - 1:
        return False
    for prev, cur in zip(intervals, intervals[1:]):
        if cur != prev and cur[0] != prev[1] + 1:
            return False
    return True


def brute_force(t_teacher, t_student, n_devices, comm=None):
    """Minimum over every valid distribution.  Returns (bottleneck, intervals per device)."""
    n_blocks = len(t_teacher[1])
    all_intervals = [(a, b) for a in range(n_blocks) for b in range(a, n_blocks)]
    best = (float("inf"), None)
    for intervals in itertools.product(all_intervals, repeat=n_devices):
        if not is_valid(intervals, n_blocks):
            continue
        worst, ok = 0.0, True
        for iv in set(intervals):
            d = intervals.count(iv)
            if d not in t_teacher:
                ok = False
                break
            worst = max(worst, device_seconds(t_teacher, t_student, iv[0], iv[1], d, comm))
        if ok and worst < best[0]:
            best = (worst, intervals)
    return best


def simulate(groups, t_teacher, t_student, steps, comm=None):
    """Event-by-event run of `steps` training steps of a schedule [(first, last, d)].

    Per step, a group runs its teacher blocks in order on the activation relayed from the group
    before it, sends the last one on as soon as it exists (the transfer itself is taken as free,
    Sec. IV-A), then trains its student blocks and updates them at once with no barrier across
    groups (Sec. IV-B).  A group starts step s when its own step s-1 is done and the activation of
    step s has arrived.  Returns the time at which the last group finishes the last step."""
    done = [0.0] * len(groups)        # when each group finished its previous step
    for _ in range(steps):
        arrived = 0.0                 # group 0 reads its input from the data loader
        for g, (first, last, d) in enumerate(groups):
            t = max(done[g], arrived)
            for i in range(first, last + 1):
                t += t_teacher[d][i]
            arrived = t
            for i in range(first, last + 1):
                t += t_student[d][i]
            if comm is not None:
                t += comm(first, last, d)
            done[g] = t
    return max(done)
