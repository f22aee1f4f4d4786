"""CPU property tests of the rollout scheduling model (Sections 3.3, 5.1.1, 5.1.2): the bound of
Proposition 1 holds on it, and the two effects the paper measures have the direction and the growth
it reports (their size depends on the paper's models and data and is not reproduced)."""
import numpy as np

from paper_2510_11345_amd import scheduler_sim as sim


def _const_engine(slots=1):
    # every step costs the same whatever the batch: generation time = number of tokens
    return sim.EngineModel(slots=slots, n_layers=1, kv_bytes_per_token=0.0, launch_s=1.0, sample_floor_s=0.0,
                           sample_per_row_s=0.0, weight_bytes=0.0)


def test_step_time_closed_form_equals_the_sum_of_steps():
    m = sim.EngineModel()
    B, L = 37, 12345.0
    want = sum(m.steps_time(1, B, L + i * B) for i in range(50))
    assert abs(m.steps_time(50, B, L) - want) <= 1e-12 * want
    # the measured points the defaults were fitted to (config 2 and config 4, one layer, attention only)
    one = sim.EngineModel(n_layers=1, sample_floor_s=0.0, sample_per_row_s=0.0, weight_bytes=0.0)
    assert abs(one.steps_time(1, 256, 888066 - 256) - 0.289e-3) < 0.01e-3
    assert abs(one.steps_time(1, 256, 471369 - 256) - 0.156e-3) < 0.01e-3


def test_proposition_1_bound_on_the_simulator():
    # K workers with one slot each and a constant step time: generation time of a sample is its length
    for seed in range(10):
        tasks = sim.draw_tasks(50, 4, seed)
        lens = np.array([t.gen_len for t in tasks], float)
        for K in (1, 4, 32):
            T = sim.run_queue(tasks, K, _const_engine())
            assert T <= len(tasks) / K * lens.mean() + lens.max() + 1e-6
            assert T >= lens.sum() / K - 1e-6
            assert sim.run_batch(tasks, K, _const_engine()) >= lens.sum() / K - 1e-6


def test_one_engine_all_slots_is_the_longest_request():
    tasks = sim.draw_tasks(8, 8, 3)
    T = sim.run_queue(tasks, 1, _const_engine(slots=64))
    assert abs(T - max(t.gen_len for t in tasks)) < 1e-9


def test_queue_scheduling_beats_batch_rollout_under_filtering_and_redundancy_helps():
    model = sim.EngineModel(slots=256)      # room for the 8 + 16 prompts of 8 responses each
    k, need, K = 8, 8, 1
    ratios0, ratios16 = [], []
    for seed in range(6):
        tasks = sim.draw_tasks(400, k, seed)
        tb = sim.filtered_rollout_time(tasks, need, k, K, model, "batch")
        t0 = sim.filtered_rollout_time(tasks, need, k, K, model, "queue", extra_prompts=0)
        t16 = sim.filtered_rollout_time(tasks, need, k, K, model, "queue", extra_prompts=16)
        ratios0.append(tb / t0)
        ratios16.append(tb / t16)
    # queue scheduling alone gains (rewards are looked at as prompts finish, no second full round is
    # waited for), redundant prompts gain more (Section 5.1.1 reports 3.4x at 8 x 8 with 16 extra)
    assert np.mean(ratios0) > 1.1
    assert np.mean(ratios16) > np.mean(ratios0) * 1.2
    assert np.mean(ratios16) > 1.5


def test_prompt_replication_gains_grow_with_scale():
    model = sim.EngineModel(slots=64)
    K = 8

    def speedup(num_prompts, n):
        r = []
        for seed in range(5):
            tasks = sim.draw_tasks(num_prompts, n, 100 + seed)
            r.append(sim.run_pinned_prompts(tasks, K, model) / sim.run_queue(tasks, K, model))
        return float(np.mean(r))

    by_batch = [speedup(b, 16) for b in (4, 16, 64)]
    by_n = [speedup(16, n) for n in (4, 16, 64)]
    # never slower; little to gain at small scale, more beyond (Section 5.1.2: up to 1.84x / 1.95x)
    assert all(s >= 0.99 for s in by_batch + by_n)
    assert by_batch[2] > by_batch[0] and by_n[2] > by_n[0]
    assert max(by_batch) > 1.15 and max(by_n) > 1.15
