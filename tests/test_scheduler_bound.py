"""CPU property test: the slot scheduler of the refill workload obeys the generation-time bound
of Proposition 1 (Section 3.3): Q tasks on K workers that each take the next task as soon as they
are free finish within (Q / K) * mean + longest."""
import numpy as np

from paper_2510_11345_amd import workloads as wl


def simulate(durations, K):
    """Queue scheduling: K slots, each takes the next task when free. Returns the makespan."""
    free_at = np.zeros(K)
    for d in durations:
        i = int(np.argmin(free_at))
        free_at[i] += d
    return free_at.max()


def test_queue_scheduling_respects_proposition_1():
    for seed in range(20):
        plan = wl.draw_refill_plan(32, 400, seed)
        lengths = plan.target_len.astype(np.float64)       # generation time in decode steps
        for K in (1, 8, 32, 256):
            T = simulate(lengths, K)
            bound = len(lengths) / K * lengths.mean() + lengths.max()
            assert T <= bound + 1e-9
            assert T >= lengths.sum() / K - 1e-9            # and cannot beat perfect packing


def test_refill_plan_shapes():
    plan = wl.draw_refill_plan(256, 1000, 0)
    assert plan.prompt_len.min() >= 128 and plan.prompt_len.max() <= 1024
    assert plan.target_len.min() >= 16 and plan.target_len.max() <= 16384
    assert (plan.start_generated[:256] < plan.target_len[:256]).all()
    assert not plan.start_generated[256:].any()
    med = np.median(wl.draw_refill_plan(256, 20000, 1).target_len)
    assert 1300 < med < 1700
