"""CPU model of rollout scheduling on K decode engines (ROLL Flash, arXiv 2510.11345, Sections 3.3,
5.1.1 and 5.1.2): batch rollout against queue scheduling, with and without redundant prompts under
dynamic filtering, and prompt replication against responses pinned to their prompt's engine.

An engine is one GPU running the decode step of this library over its running requests (continuous
batching with a fixed number of slots).  Every running request gains one token per step, and a step
costs what this library's kernels were measured to cost for that batch on an MI355X:

    t_step(B, sum_L) = weight_bytes / bandwidth
                       + n_layers * (t_launch + kv_bytes_per_token * sum_L / bandwidth) + t_sample(B)

(the attention launches and the sampling launch as measured; the projection and MLP GEMMs of a real
model are not part of this library and enter only as the time to stream the weights once per step at
the same bandwidth, which is what they cost at decode batch sizes and what makes a few more
concurrent requests nearly free at small batches.  Absolute times are therefore not a model's; the
scheduling effects, which come from the length distribution, are what is modelled.)  Between two finishes all
running requests advance in lockstep, so the simulation jumps from finish to finish and sums the
step times in closed form.

Nothing here runs on the GPU and nothing of it is on the decode path; tests/test_scheduler_sim.py
checks the bound of Proposition 1 on it and the direction and growth of the two effects.
"""
from __future__ import annotations

import dataclasses
import heapq
import math
from typing import List, Optional, Sequence

import numpy as np


@dataclasses.dataclass(frozen=True)
class EngineModel:
    """Step-time model of one engine.  Defaults: the 7B-class shape (config 2 / 4) as measured:
    a fused attention launch takes ~3.6 us + 158 us per GB of live KV (0.289 ms at 1.81 GB, 0.156 ms
    at 0.97 GB), the sampling launch 36 us up to 256 rows and ~0.13 us per row beyond."""
    slots: int = 256
    n_layers: int = 28
    kv_bytes_per_token: float = 2048.0      # K and V, bf16, 4 KV heads x 128, one layer
    launch_s: float = 3.6e-6
    bandwidth_Bps: float = 6.33e12
    sample_floor_s: float = 36e-6
    sample_per_row_s: float = 0.13e-6
    weight_bytes: float = 15.2e9            # a 7B-class model in bf16, streamed once per step

    def steps_time(self, m: int, B: int, sum_L: float) -> float:
        """Seconds for m consecutive steps that start with B running requests holding sum_L tokens
        (each step adds one token to every request)."""
        if m <= 0 or B <= 0:
            return 0.0
        per_step_fixed = (self.weight_bytes / self.bandwidth_Bps + self.n_layers * self.launch_s +
                          max(self.sample_floor_s, self.sample_per_row_s * B))
        tokens_read = m * sum_L + B * m * (m + 1) / 2.0
        return m * per_step_fixed + self.n_layers * self.kv_bytes_per_token * tokens_read / self.bandwidth_Bps


@dataclasses.dataclass
class Task:
    """One response to generate: prompt tokens already in the cache when it starts, tokens to decode."""
    prompt_len: int
    gen_len: int
    prompt_id: int = 0
    reward: int = 0


class _Engine:
    """Running requests of one engine as (finish step count, tokens at admission) pairs, advanced in
    lockstep; `clock` in seconds, `steps` in decode steps since the start."""

    def __init__(self, model: EngineModel):
        self.model = model
        self.clock = 0.0
        self.steps = 0
        self.running: List[tuple] = []      # heap of (finish_step, seq, task)
        self.sum_L = 0.0                     # tokens held by the running requests now
        self._seq = 0

    def free_slots(self) -> int:
        return self.model.slots - len(self.running)

    def admit(self, task: Task) -> None:
        heapq.heappush(self.running, (self.steps + max(task.gen_len, 1), self._seq, task))
        self._seq += 1
        self.sum_L += task.prompt_len

    def catch_up(self, now: float) -> None:
        """Advance to the last step boundary at or before `now` (no request finishes on the way: the
        caller handles finishes in time order), so that a request admitted at `now` joins there."""
        if not self.running:
            self.clock = max(self.clock, now)
            return
        B, lo, hi = len(self.running), 0, self.running[0][0] - self.steps - 1
        while lo < hi:                       # largest m with clock + steps_time(m) <= now
            mid = (lo + hi + 1) // 2
            if self.clock + self.model.steps_time(mid, B, self.sum_L) <= now:
                lo = mid
            else:
                hi = mid - 1
        if lo > 0:
            self.clock += self.model.steps_time(lo, B, self.sum_L)
            self.steps += lo
            self.sum_L += B * lo

    def next_finish_time(self) -> float:
        if not self.running:
            return math.inf
        m = self.running[0][0] - self.steps
        return self.clock + self.model.steps_time(m, len(self.running), self.sum_L)

    def advance_to_next_finish(self) -> List[Task]:
        m = self.running[0][0] - self.steps
        B = len(self.running)
        self.clock += self.model.steps_time(m, B, self.sum_L)
        self.steps += m
        self.sum_L += B * m
        done = []
        while self.running and self.running[0][0] == self.steps:
            _, _, t = heapq.heappop(self.running)
            self.sum_L -= t.prompt_len + max(t.gen_len, 1)
            done.append(t)
        return done

    def abort_all(self) -> None:
        self.running.clear()
        self.sum_L = 0.0


def run_queue(tasks: Sequence[Task], K: int, model: EngineModel, stop=None, in_flight: Optional[int] = None) -> float:
    """Queue scheduling: a task starts as soon as any engine has a free slot.  `in_flight` caps the
    tasks started and not finished (None: the engines' slots).  `stop(task)` is called at every finish
    and ends the run (everything still running is aborted) when it returns True.  Returns the
    completion time in seconds."""
    engines = [_Engine(model) for _ in range(K)]
    cap = K * model.slots if in_flight is None else in_flight
    nxt, active, now = 0, 0, 0.0

    def refill():
        nonlocal nxt, active
        while nxt < len(tasks) and active < cap:
            e = max(engines, key=lambda g: g.free_slots())      # least loaded engine
            if e.free_slots() <= 0:
                break
            e.catch_up(now)
            e.admit(tasks[nxt])
            nxt += 1
            active += 1

    refill()
    while active:
        e = min(engines, key=lambda g: g.next_finish_time())
        for t in e.advance_to_next_finish():
            active -= 1
            now = e.clock
            if stop is not None and stop(t):
                for g in engines:
                    g.abort_all()
                return now
        now = e.clock
        refill()
    return now


def run_batch(tasks: Sequence[Task], K: int, model: EngineModel) -> float:
    """Batch rollout: the tasks are dealt to the engines up front (task i to engine i mod K), every
    engine works through its share, and the step ends when the slowest engine is done."""
    return max(run_queue(tasks[k::K], 1, model) for k in range(K)) if tasks else 0.0


def run_pinned_prompts(tasks: Sequence[Task], K: int, model: EngineModel) -> float:
    """No prompt replication (Section 5.1.2): a prompt with n responses is one request to one engine
    (prompts dealt round-robin), which decodes the n responses together and gives their n slots back
    only when the longest of them is done; the step ends when the slowest engine is done."""
    by_prompt = {}
    for t in tasks:
        by_prompt.setdefault(t.prompt_id, []).append(t)
    shares = [[] for _ in range(K)]
    for i, pid in enumerate(sorted(by_prompt)):
        shares[i % K].append(by_prompt[pid])
    worst = 0.0
    for groups in shares:
        e, nxt, held, left = _Engine(model), 0, 0, {}
        while nxt < len(groups) or e.running:
            while nxt < len(groups) and e.free_slots() - held >= len(groups[nxt]):
                for t in groups[nxt]:
                    e.admit(t)
                left[groups[nxt][0].prompt_id] = len(groups[nxt])
                nxt += 1
            if not e.running:          # a prompt with more responses than the engine has slots
                raise ValueError("a prompt's responses do not fit the engine's slots")
            for t in e.advance_to_next_finish():
                left[t.prompt_id] -= 1
                if left[t.prompt_id]:
                    held += 1                                        # slot stays with its prompt
                else:
                    held -= len(by_prompt[t.prompt_id]) - 1          # the whole prompt is done
        worst = max(worst, e.clock)
    return worst


def draw_tasks(num_prompts: int, responses_per_prompt: int, seed: int, median_len: float = 1500.0,
               sigma: float = 1.0, clip=(16, 16384), prompt_range=(128, 1024)) -> List[Task]:
    """Long-tailed response lengths (lognormal, the law of the refill workload) and, per prompt, a pass
    rate drawn from Beta(0.5, 0.5) that decides each response's 0/1 reward: many prompts are nearly
    always or nearly never solved, which is what dynamic filtering throws away."""
    rng = np.random.default_rng([seed, 0x53434844])
    tasks = []
    for p in range(num_prompts):
        plen = int(rng.integers(prompt_range[0], prompt_range[1] + 1))
        rate = float(rng.beta(0.5, 0.5))
        for _ in range(responses_per_prompt):
            g = int(np.clip(np.rint(np.exp(rng.normal(math.log(median_len), sigma))), clip[0], clip[1]))
            tasks.append(Task(plen, g, p, int(rng.random() < rate)))
    return tasks


def filtered_rollout_time(tasks: Sequence[Task], need_prompts: int, responses_per_prompt: int, K: int,
                          model: EngineModel, mode: str, extra_prompts: int = 0) -> float:
    """Time until `need_prompts` prompts have all their responses and a non-zero reward variance within
    the group (Section 5.1.1's dynamic filtering).
    mode "batch": rounds of need_prompts prompts, each a batch rollout whose rewards are looked at
      only when the whole round is done; further rounds until enough prompts qualify.
    mode "queue": need_prompts + extra_prompts prompts in flight under queue scheduling, rewards
      looked at when a prompt's last response finishes, everything aborted once enough qualify."""
    k = responses_per_prompt
    groups = {}
    for t in tasks:
        groups.setdefault(t.prompt_id, []).append(t)
    order = sorted(groups)
    qualifies = {p: 0 < sum(t.reward for t in groups[p]) < k for p in order}
    if mode == "batch":
        total, got, pos = 0.0, 0, 0
        while got < need_prompts and pos < len(order):
            chunk = order[pos:pos + need_prompts]
            pos += len(chunk)
            total += run_batch([t for p in chunk for t in groups[p]], K, model)
            got += sum(qualifies[p] for p in chunk)
        return total
    if mode != "queue":
        raise ValueError(mode)
    left = {p: k for p in order}
    state = {"got": 0}

    def stop(t: Task) -> bool:
        left[t.prompt_id] -= 1
        if left[t.prompt_id] == 0 and qualifies[t.prompt_id]:
            state["got"] += 1
        return state["got"] >= need_prompts

    flat = [t for p in order for t in groups[p]]
    return run_queue(flat, K, model, stop=stop, in_flight=(need_prompts + extra_prompts) * k)
