"""Host model of the rendezvous of the switched-off split kernel (csrc/zp_split.h), CPU only.

The split kernel lets C workgroups share a unit: each draws a ticket when it STARTS (one counter per ticket stream),
works on its chunk, raises the unit's arrival count, and all but the last arriver wait for the unit's ready flag.  On
MI355X that bounded wait has expired now and then.  This model checks the part that can be checked without a GPU:
with a dispatcher that hands out workgroups strictly in order, a fixed number of resident slots per XCD (workgroup i
goes to XCD i mod 8 and must wait for a slot THERE: head-of-line blocking), and arbitrary durations, the protocol can
never leave every resident workgroup waiting, and the number of workgroups waiting for peers that have not started stays
within NS x (C - 1).  It runs the two launch shapes whose wait expired (a 14B-like one with C = 33 and two ticket
streams, an 8B-like one with C = 17 and four) and smaller adversarial ones.  A deadlock in the model would name a
cause for the expiry; none is found, which leaves the visibility of the exchanged words across XCDs as the open suspect.
"""
import heapq

import numpy as np
import pytest


def simulate(units, C, NS, slots_per_xcd, seed, n_xcd=8, tail_scale=8.0):
    """Event-driven run of the protocol.  Returns (finished units, peak waiters-for-unstarted-peers, deadlocked)."""
    rng = np.random.default_rng(seed)
    grid = units * C
    ticket = [0] * NS
    arrive1 = [0] * units
    started = [0] * units              # members of the unit that have drawn a ticket
    ready = [False] * units
    arrive2 = [0] * units
    waiting = {}                       # unit -> list of (workgroup, xcd) blocked on its ready flag
    free = [slots_per_xcd] * n_xcd
    events = []                        # (time, seq, kind, workgroup, unit, xcd)
    seq = 0
    now = 0.0
    next_bid = 0
    done_units = 0
    peak = 0

    def push(t, kind, wg, unit, x):
        nonlocal seq
        heapq.heappush(events, (t, seq, kind, wg, unit, x))
        seq += 1

    def dispatch():
        # strictly in order: the head of the queue waits for a slot on ITS xcd and blocks everything behind it
        nonlocal next_bid
        while next_bid < grid:
            x = next_bid % n_xcd
            if free[x] == 0:
                return
            free[x] -= 1
            bid = next_bid
            next_bid += 1
            xs = bid % NS
            t = ticket[xs]
            ticket[xs] += 1
            unit = xs + NS * (t // C)
            if unit >= units:          # more workgroups than work in this stream: leaves at once
                free[x] += 1
                continue
            started[unit] += 1
            push(now + rng.exponential(1.0), "phase1_done", bid, unit, x)

    dispatch()
    while events:
        now, _, kind, wg, unit, x = heapq.heappop(events)
        if kind == "phase1_done":
            arrive1[unit] += 1
            if arrive1[unit] == C:     # last arriver combines, publishes, goes on; the waiters follow
                ready[unit] = True
                push(now + rng.exponential(0.2), "phase2_done", wg, unit, x)
                for w2, x2 in waiting.pop(unit, []):
                    push(now + rng.exponential(0.2), "phase2_done", w2, unit, x2)
            else:
                waiting.setdefault(unit, []).append((wg, x))
        elif kind == "phase2_done":
            arrive2[unit] += 1
            if arrive2[unit] == C:     # the finisher runs selection and compaction alone: long
                push(now + rng.exponential(tail_scale), "exit", wg, unit, x)
                done_units += 1
            else:
                push(now, "exit", wg, unit, x)
        else:
            free[x] += 1
            dispatch()
        # workgroups blocked on a unit some of whose members have not even started
        blocked = sum(len(v) for u_, v in waiting.items() if started[u_] < C)
        peak = max(peak, blocked)
    deadlocked = bool(waiting) or next_bid < grid
    return done_units, peak, deadlocked


@pytest.mark.parametrize("units,C,NS,slots", [
    (2048, 33, 2, 32),      # 14B-like launch shape whose wait expired (one 8-wave workgroup per CU)
    (2048, 17, 4, 64),      # 8B-like launch shape whose wait expired (two per CU)
    (64, 17, 4, 9),         # barely enough slots: 8 x 9 = 72 resident workgroups for 4 x 16 possible waiters
    (40, 33, 2, 9),
    (37, 5, 1, 1),          # one slot per XCD: 8 resident workgroups, at most 4 waiters
    (24, 8, 8, 8),          # one stream per XCD
])
def test_rendezvous_never_deadlocks_and_waiters_stay_bounded(units, C, NS, slots):
    assert units % NS == 0 or NS == 1
    for seed in range(5):
        done, peak, dead = simulate(units, C, NS, slots, seed)
        assert not dead, "deadlock in the model: units=%d C=%d NS=%d slots=%d seed=%d" % (units, C, NS, slots, seed)
        assert done == units
        assert peak <= NS * (C - 1)


def test_model_does_deadlock_when_the_waiter_bound_exceeds_the_chip():
    """The model is not vacuous: with fewer resident slots than possible waiters it does lock up."""
    locked = 0
    for seed in range(10):
        _, _, dead = simulate(units=32, C=17, NS=4, slots_per_xcd=2, seed=seed)   # 16 slots, up to 64 waiters
        locked += dead
    assert locked > 0
