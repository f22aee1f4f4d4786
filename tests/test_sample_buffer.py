"""CPU property tests of the SampleBuffer's asynchronous-ratio rules (Section 4.3 of the paper):
capacity (1 + alpha) * batch, per-sample freshness n - init <= alpha, nothing dropped; and an
event-driven rollout / train simulation on top of it (queue scheduling over K slots, long-tailed
generation times) that checks the invariants on every event and that asynchrony shortens the
run without breaking them."""
import heapq

import numpy as np
import pytest

from paper_2510_11345_amd import binding as rb
from paper_2510_11345_amd import workloads as wl


def test_capacity_and_errors():
    b = rb.SampleBuffer(4, 1.5)
    assert b.capacity == 10 and b.version == 0
    tickets = [b.begin()[0] for _ in range(8)]
    assert b.begin() is None and b.outstanding == 8          # a 9th would be consumed 2 versions ahead
    assert b.take_batch() is None                            # nothing complete yet
    with pytest.raises(rb.RollError):
        b.complete(999)
    b.abort(tickets[0])
    with pytest.raises(rb.RollError):
        b.complete(tickets[0])                               # interrupted, must be resumed first
    assert b.resume(tickets[0]) == 0
    for t in tickets[:4]:
        b.complete(t, payload=100 + t)
    got = b.take_batch()
    assert [g[0] for g in got] == tickets[:4] and [g[2] for g in got] == [100, 101, 102, 103]
    assert b.outstanding == 4
    assert b.begin() is None                                 # the trainer holds this version's batch: 1 + 4 // 4 > 1.5
    assert b.advance_version() and b.begin() is not None
    with pytest.raises(rb.RollError):
        rb.SampleBuffer(0, 1.0)
    with pytest.raises(rb.RollError):
        rb.SampleBuffer(4, -0.5)


def test_alpha_zero_is_synchronous():
    b = rb.SampleBuffer(3, 0.0)
    ts = [b.begin()[0] for _ in range(3)]
    assert b.begin() is None
    assert not b.advance_version()          # samples of version 0 must be consumed before version 1
    for t in ts:
        b.complete(t)
    assert all(v == 0 for _, v, _ in b.take_batch())
    assert b.advance_version() and b.version == 1
    assert b.begin()[1] == 1


def test_due_samples_block_the_trainer_instead_of_going_stale():
    b = rb.SampleBuffer(2, 1.0)             # capacity 4
    ts = [b.begin()[0] for _ in range(4)]   # all initiated at version 0
    b.complete(ts[2]); b.complete(ts[3])
    got = b.take_batch()                    # version 0: nothing is due yet, the two finished ones go
    assert [g[0] for g in got] == [ts[2], ts[3]]
    assert b.begin() is None                # 1 + 2 // 2 batches ahead > alpha
    assert b.advance_version()              # -> 1; ts[0], ts[1] are now due (they cannot see version 2)
    n1 = b.begin()[0]; n2 = b.begin()[0]
    b.complete(n1); b.complete(n2)
    assert b.take_batch() is None           # two complete, but the due stragglers come first
    assert not b.advance_version()
    b.complete(ts[0]); b.complete(ts[1])
    got = b.take_batch()
    assert [g[0] for g in got] == [ts[0], ts[1]] and all(b.version - v <= 1 for _, v, _ in got)


def simulate(alpha, batch, K, n_steps, seed, train_time=40.0, abort_on_update=False):
    """Rollout on K slots with queue scheduling + trainer, driven by the buffer's rules.
    Generation time of a sample = its response length in decode steps (long-tailed).
    Returns (makespan, max_gap, consumed, log of invariant checks)."""
    rng = np.random.default_rng(seed)
    plan = wl.draw_refill_plan(K, 100000, seed, target_median=120.0, target_clip=(4, 4000))
    buf = rb.SampleBuffer(batch, alpha)
    now, events, free_slots, next_len = 0.0, [], K, 0
    remaining = {}                                   # ticket -> remaining generation time
    running = {}                                     # ticket -> finish time
    training, steps_done, max_gap, consumed, begun = False, 0, 0, 0, 0

    def start_more():
        nonlocal free_slots, next_len, begun
        # resume reclaimed samples first, then start new ones while the buffer allows
        for t in [t for t in list(remaining) if t not in running]:
            if free_slots == 0:
                return
            buf.resume(t)
            running[t] = now + remaining[t]; heapq.heappush(events, (running[t], "gen", t)); free_slots -= 1
        while free_slots > 0:
            r = buf.begin()
            if r is None:
                return
            t = r[0]; begun += 1
            remaining[t] = float(plan.target_len[next_len]); next_len += 1
            running[t] = now + remaining[t]; heapq.heappush(events, (running[t], "gen", t)); free_slots -= 1

    start_more()
    while steps_done < n_steps:
        assert buf.outstanding <= buf.capacity
        if not training:
            got = buf.take_batch()
            if got is not None:
                for _, v, _ in got:
                    gap = buf.version - v
                    assert gap <= alpha + 1e-12
                    max_gap = max(max_gap, gap)
                consumed += len(got)
                training = True
                heapq.heappush(events, (now + train_time, "train", -1))
                start_more()
                continue
        if not events:
            raise AssertionError("deadlock: nothing running and the trainer cannot proceed")
        now, kind, t = heapq.heappop(events)
        if kind == "gen":
            if running.get(t) != now:
                continue                              # stale event of an aborted run
            del running[t]; del remaining[t]
            buf.complete(t); free_slots += 1
            start_more()
        else:                                         # train step done: model update
            assert buf.advance_version(), "a sample would exceed alpha: the rules failed"
            training = False
            steps_done += 1
            if abort_on_update:                       # suspend -> ABORT everything running -> resume
                for t2, fin in list(running.items()):
                    remaining[t2] = fin - now
                    buf.abort(t2); del running[t2]; free_slots += 1
            start_more()
    return now, max_gap, consumed, begun, buf.outstanding


@pytest.mark.parametrize("alpha", [0.0, 1.0, 2.0, 0.5])
@pytest.mark.parametrize("abort_on_update", [False, True])
def test_invariants_hold_in_simulation(alpha, abort_on_update):
    for seed in range(3):
        t, max_gap, consumed, begun, left = simulate(alpha, batch=16, K=24, n_steps=30, seed=seed,
                                                     abort_on_update=abort_on_update)
        assert consumed == 30 * 16
        assert begun == consumed + left              # nothing was dropped: begun = taken + still outstanding
        assert max_gap <= alpha


def test_asynchrony_shortens_the_run():
    sync = np.mean([simulate(0.0, 16, 24, 30, s)[0] for s in range(4)])
    async2 = np.mean([simulate(2.0, 16, 24, 30, s)[0] for s in range(4)])
    async1 = np.mean([simulate(1.0, 16, 24, 30, s)[0] for s in range(4)])
    assert async1 < 0.9 * sync and async2 <= async1 * 1.02   # generation overlaps training; the long tail no longer stalls every step
