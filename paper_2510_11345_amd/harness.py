"""Device-side state of a running decode batch, built through the C ABI.

Plumbing shared by the benchmark, the smoke check and the end-to-end tests:
it owns the torch tensors (device memory only), drives the allocator and
calls the library once per step.  No arithmetic of the decode step is here.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as rb
from . import workloads as wl


class DecodeBatch:
    """A batch of `cfg.batch` slots whose KV lives in paged pools.

    The pools are filled with i.i.d. N(0,1) bf16 once (a slot's "history" is
    whatever its pages hold); lengths are grown through roll_kv_alloc_batch in
    page-sized rounds over all rows, so that the physical pages of different
    rows interleave the way they do in a long-running continuous batch.
    """

    def __init__(self, cfg: wl.DecodeConfig, seed: int, lengths: np.ndarray, headroom_tokens: int = 0,
                 out_dtype=torch.bfloat16, device: str = "cuda",
                 spare_pages: int = 64, max_len: int | None = None, fill_pools: bool = True,
                 profile_events: bool = False, num_pages: int | None = None, fused: bool = True,
                 side_by_side: bool = True, run_pages: int | None = None):
        self.cfg, self.seed, self.device = cfg, seed, device
        B, P = cfg.batch, cfg.page_size
        Hq, Hkv, D = cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim
        lengths = np.asarray(lengths, dtype=np.int64)
        assert len(lengths) == B
        cap = int(max(int(lengths.max()) + headroom_tokens, 1)) if max_len is None else int(max_len)
        self.max_pages = (cap + P - 1) // P
        # pages are handed out in aligned runs that cover one 32-token step of the attention kernel
        self.run_pages = max(1, 32 // P) if run_pages is None else int(run_pages)
        R = self.run_pages
        need = int((((np.minimum(lengths + headroom_tokens, cap) + P - 1) // P + R - 1) // R * R).sum())
        self.num_pages = (need + spare_pages + R - 1) // R * R if num_pages is None else int(num_pages)
        self.page_table = torch.empty((B, self.max_pages), dtype=torch.int32, device=device)
        self.seq_lens = torch.zeros((B,), dtype=torch.int32, device=device)
        self.pool = rb.KvPool(self.num_pages, P, B, self.max_pages, self.page_table, self.seq_lens, run_pages=R)
        if side_by_side:
            # one allocation, the K block and the V block of a page next to each other
            both = (wl.randn_bf16((self.num_pages, 2, Hkv * P * D), seed, 2, device) if fill_pools else
                    torch.zeros((self.num_pages, 2, Hkv * P * D), dtype=torch.bfloat16, device=device))
            self.k_pages = both[:, 0].view(self.num_pages, Hkv, D // 8, P, 8)
            self.v_pages = both[:, 1].view(self.num_pages, Hkv, P // 8, D, 8)
        elif fill_pools:
            self.k_pages = wl.randn_bf16((self.num_pages, Hkv, D // 8, P, 8), seed, 2, device)
            self.v_pages = wl.randn_bf16((self.num_pages, Hkv, P // 8, D, 8), seed, 3, device)
        else:
            self.k_pages = torch.zeros((self.num_pages, Hkv, D // 8, P, 8), dtype=torch.bfloat16, device=device)
            self.v_pages = torch.zeros((self.num_pages, Hkv, P // 8, D, 8), dtype=torch.bfloat16, device=device)
        self.q = wl.randn_bf16((B, Hq, D), seed, 1, device)
        self.k_new = wl.randn_bf16((B, Hkv, D), seed, 5, device)
        self.v_new = wl.randn_bf16((B, Hkv, D), seed, 6, device)
        self.out = torch.zeros((B, Hq, D), dtype=out_dtype, device=device)
        self.tokens = torch.zeros((B,), dtype=torch.int32, device=device)
        self.logprob = torch.zeros((B,), dtype=torch.float32, device=device)
        self.lengths = np.zeros(B, dtype=np.int64)
        self.all_slots = np.arange(B, dtype=np.int32)
        self.ones = np.ones(B, dtype=np.int32)
        self.ev_pairs = []   # (begin, end, sum of seq_lens) per profiled step
        self.ev_spare = []   # pre-created event pairs, so that none is created inside a timed loop
        self.profile_events = profile_events
        self.fused = fused
        self.out_dtype = out_dtype
        self.desc = rb.attn_desc(self.q, self.k_pages, self.page_table, P, out_dtype)
        self._ws = rb.new_attn_workspace(self.desc, device)
        self.grow_to(lengths)

    # -- allocator ------------------------------------------------------------
    def grow_to(self, target: np.ndarray) -> None:
        """Grow every row to its target length, one page-sized round over all rows at a time."""
        target = np.asarray(target, dtype=np.int64)
        P = self.cfg.page_size
        while True:
            todo = np.flatnonzero(self.lengths < target)
            if len(todo) == 0:
                break
            n = np.minimum(target[todo] - self.lengths[todo], P).astype(np.int32)
            rb.roll_kv_alloc_batch(self.pool, todo.astype(np.int32), n)
            self.lengths[todo] += n
        rb.roll_kv_commit(self.pool)

    def total_tokens(self) -> int:
        return int(self.lengths.sum())

    # -- one decode step --------------------------------------------------------
    def step(self, logits: torch.Tensor, step_index: int, temperature=None, top_p=None,
             grow: bool = True) -> None:
        """alloc (+1 token per row) -> commit + append K/V + attention (one launch when self.fused,
        else two) -> sample."""
        cfg = self.cfg
        fused = grow and self.fused
        if grow:
            rb.roll_kv_alloc_batch(self.pool, self.all_slots, self.ones)
            self.lengths += 1
            if not fused:
                rb.roll_kv_commit_append(self.pool, self.k_new, self.v_new, self.k_pages, self.v_pages)
        desc = self.desc
        if self.profile_events:
            e0, e1 = self.ev_spare.pop() if self.ev_spare else (rb.ProfEvent(), rb.ProfEvent())
            rb.roll_prof_attn_events(e0, e1)
            self.ev_pairs.append((e0, e1, self.total_tokens()))
        if fused:
            rb.roll_decode_step_attn(self.pool, self.k_new, self.v_new, self.q, self.k_pages, self.v_pages,
                                     self.out, desc, self._ws)
        else:
            rb.roll_decode_attn(self.q, self.k_pages, self.v_pages, self.page_table, self.seq_lens, self.out,
                                desc, self._ws)
        if self.profile_events:
            rb.roll_prof_attn_events(None, None)
        sdesc = rb.sample_desc(logits)
        rb.roll_sample_logprob(logits, cfg.temperature if temperature is None else temperature,
                               cfg.top_p if top_p is None else top_p, self.seed, step_index,
                               self.tokens, self.logprob, sdesc, None)

    def pages_held(self) -> int:
        """Pages that the slots hold, counting the unused rest of every slot's last run."""
        R = self.run_pages
        return sum((len(rb.roll_kv_slot_pages(self.pool, s)) + R - 1) // R * R for s in range(self.cfg.batch))

    # -- host copies for the oracle --------------------------------------------
    def gather_rows(self, rows):
        """Host copy of the listed rows: compact pools holding only their pages and a remapped
        page table; returns (q_bits, k_bits, v_bits, page_table, seq_lens) over len(rows) rows."""
        P = self.cfg.page_size
        pages, table = [], np.full((len(rows), self.max_pages), -1, dtype=np.int32)
        for i, r in enumerate(rows):
            pr = rb.roll_kv_slot_pages(self.pool, int(r))
            table[i, :len(pr)] = np.arange(len(pages), len(pages) + len(pr))
            pages.extend(pr)
        idx = torch.tensor(pages, dtype=torch.int64, device=self.device)
        k = wl.bits(self.k_pages.index_select(0, idx)).reshape(-1)
        v = wl.bits(self.v_pages.index_select(0, idx)).reshape(-1)
        q = wl.bits(self.q[torch.tensor(list(rows), device=self.device)])
        lens = self.lengths[list(rows)].astype(np.int32)
        return q, k, v, table, lens

    def close(self):
        self.pool.close()


class RefillLoop:
    """Queue-scheduled continuous refill on top of a DecodeBatch: every slot holds a request with
    a pre-drawn target length; a slot whose request has finished is released and at once given
    the next prompt of the queue, which is prefilled into freshly allocated pages (all prompts
    of a tick in one roll_prefill_attn call; with prefill=False only their K/V is written);
    then every slot decodes one token.  Prompt Q/K/V are slices of a seeded random bank."""

    def __init__(self, cfg: wl.DecodeConfig, plan: wl.RefillPlan, seed: int, max_len: int,
                 out_dtype=torch.bfloat16, device: str = "cuda", prefill: bool = True,
                 side_by_side: bool = True, run_pages: int | None = None):
        self.cfg, self.plan, self.seed, self.device = cfg, plan, seed, device
        self.prefill = prefill
        self.bank_tokens = int(plan.prompt_len.max()) + 4096
        self.bank_q = wl.randn_bf16((self.bank_tokens, cfg.num_q_heads, cfg.head_dim), seed, 1000, device)
        self.bank_k = wl.randn_bf16((self.bank_tokens, cfg.num_kv_heads, cfg.head_dim), seed, 1001, device)
        self.bank_v = wl.randn_bf16((self.bank_tokens, cfg.num_kv_heads, cfg.head_dim), seed, 1002, device)
        self.last_prefill = None   # (q, out, [(slot, n, first token)]) of the latest tick with refills
        # chunk arrays travel through a small ring of pinned buffers (asynchronous copies, so the
        # host keeps running ahead of the GPU; an event per buffer guards its reuse)
        self._ring = [dict(host=torch.zeros((3, cfg.batch + 1), dtype=torch.int32).pin_memory(),
                           dev=torch.zeros((3, cfg.batch + 1), dtype=torch.int32, device=device), ev=None)
                      for _ in range(8)]
        self._ring_next = 0
        B = cfg.batch
        self.request = np.arange(B, dtype=np.int64)          # request id held by each slot
        self.generated = plan.start_generated[:B].astype(np.int64).copy()
        self.next_request = B
        start_len = plan.prompt_len[:B].astype(np.int64) + self.generated
        # the pool can hold every slot at max_len, so a refill never runs out of pages
        R = max(1, 32 // cfg.page_size) if run_pages is None else int(run_pages)   # DecodeBatch's run length
        total_pages = B * (((max_len + cfg.page_size - 1) // cfg.page_size + R - 1) // R * R)
        self.batch = DecodeBatch(cfg, seed, start_len, out_dtype=out_dtype, device=device,
                                 max_len=max_len, fill_pools=True, num_pages=total_pages,
                                 side_by_side=side_by_side, run_pages=run_pages)
        self.refills = 0
        self.refill_log = []  # (step, slot, request)
        self.prefill_events = []  # (begin, end) around the prefill launches of a tick, while the batch profiles
        self._load_torch_kernels()

    def _load_torch_kernels(self):
        """torch loads a kernel the first time an operation needs it, which takes milliseconds:
        run once what a tick with several prompts uses (concatenation of bank slices, the
        pinned-buffer copy, an event), so that no step of a timed loop pays for it."""
        for bank in (self.bank_q, self.bank_k, self.bank_v):
            torch.cat([bank[:2], bank[1:3]])
        slot_ = self._ring[0]
        slot_["host"][0, :2] = torch.tensor([0, 0], dtype=torch.int32)
        slot_["dev"].copy_(slot_["host"], non_blocking=True)
        torch.empty((4, self.cfg.num_q_heads, self.cfg.head_dim), dtype=self.batch.out_dtype, device=self.device)
        ev = torch.cuda.Event()
        ev.record()
        ev.synchronize()

    def _prompt(self, request: int, n: int):
        """Q, K, V of a request's prompt: n consecutive tokens of the bank."""
        o = (request * 977) % (self.bank_tokens - n)
        return self.bank_q[o:o + n], self.bank_k[o:o + n], self.bank_v[o:o + n]

    def step(self, logits: torch.Tensor, step_index: int) -> list:
        """One scheduler tick + one decode step.  Returns the slots refilled at this step."""
        b, plan, cfg = self.batch, self.plan, self.cfg
        done = np.flatnonzero(self.generated >= plan.target_len[self.request])
        refilled = []
        for slot in done:
            if self.next_request >= len(plan.prompt_len):
                raise RuntimeError("prompt queue exhausted")
            rb.roll_kv_release(b.pool, int(slot))
            req = self.next_request
            self.next_request += 1
            n = int(plan.prompt_len[req])
            rb.roll_kv_alloc(b.pool, int(slot), n)
            self.request[slot], self.generated[slot] = req, 0
            b.lengths[slot] = n
            refilled.append((int(slot), req, n))
        if refilled:
            rb.roll_kv_commit(b.pool)   # the prompt writer looks its pages up on the device
            parts = [self._prompt(req, n) for _, req, n in refilled]
            # one prompt (the usual tick): its slices of the bank as they are, no copy
            q, k, v = parts[0] if len(parts) == 1 else (torch.cat([p[i] for p in parts]) for i in range(3))
            lens = [n for _, _, n in refilled]
            first = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
            if self.prefill:
                out = torch.empty((q.shape[0], cfg.num_q_heads, cfg.head_dim), dtype=b.out_dtype, device=self.device)
                slot_ = self._ring[self._ring_next]
                self._ring_next = (self._ring_next + 1) % len(self._ring)
                if slot_["ev"] is not None:
                    slot_["ev"].synchronize()
                n_ch = len(refilled)
                slot_["host"][0, :n_ch] = torch.tensor([r[0] for r in refilled], dtype=torch.int32)
                slot_["host"][1, :n_ch] = 0
                slot_["host"][2, :n_ch + 1] = torch.from_numpy(first)
                meta = slot_["dev"]
                meta.copy_(slot_["host"], non_blocking=True)
                if b.profile_events:
                    e0, e1 = rb.ProfEvent(), rb.ProfEvent()
                    e0.record()
                rb.roll_prefill_attn(q, k, v, meta[0, :n_ch], meta[1, :n_ch], meta[2, :n_ch + 1], b.k_pages,
                                     b.v_pages, b.page_table, out, cfg.page_size)
                if b.profile_events:
                    e1.record()
                    self.prefill_events.append((e0, e1))
                slot_["ev"] = torch.cuda.Event()
                slot_["ev"].record()
                self.last_prefill = (q, out, [(r[0], r[2], int(f)) for r, f in zip(refilled, first)])
            else:
                slots = torch.from_numpy(np.repeat([r[0] for r in refilled], lens).astype(np.int32)).pin_memory().to(self.device, non_blocking=True)
                pos = torch.from_numpy(np.concatenate([np.arange(n) for n in lens]).astype(np.int32)).pin_memory().to(self.device, non_blocking=True)
                rb.roll_kv_append_tokens(k, v, slots, pos, None, b.k_pages, b.v_pages, b.page_table,
                                         cfg.page_size)
            for slot, req, _ in refilled:
                self.refill_log.append((step_index, slot, req))
            self.refills += len(refilled)
        b.step(logits, step_index)      # +1 token per slot, commit + append, attention, sampling
        self.generated += 1
        return [r[0] for r in refilled]

    def close(self):
        self.batch.close()
