"""ctypes binding of libroll_decode.so: same names as the C ABI, marshalling only.

Every function takes torch tensors that already live on the GPU (PyTorch is
used for device memory and streams only), passes their pointers and the
current stream to the library and raises ``RollError`` on a non-zero status.
There is no fallback: if the library is missing or a kernel cannot run, the
call fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# ROLL_DECODE_LIB names another build of the same sources (the CPU test suite points it at a build
# whose host code is instrumented with sanitizers).
LIB_PATH = os.environ.get("ROLL_DECODE_LIB") or os.path.join(_HERE, "libroll_decode.so")

ROLL_BF16, ROLL_F32 = 0, 1

EXPORTS = [
    "roll_last_error", "roll_version",
    "roll_kv_pool_create", "roll_kv_pool_destroy", "roll_kv_alloc", "roll_kv_alloc_batch", "roll_kv_release",
    "roll_kv_commit", "roll_kv_commit_append", "roll_kv_free_pages", "roll_kv_seq_len", "roll_kv_slot_pages",
    "roll_kv_fused_steps",
    "roll_kv_append_tokens",
    "roll_decode_attn_workspace_bytes", "roll_decode_attn_workspace_init", "roll_decode_attn_workspace_check",
    "roll_decode_attn", "roll_decode_attn_static", "roll_decode_attn_ranges",
    "roll_decode_step_attn", "roll_prefill_attn",
    "roll_sample_logprob_workspace_bytes", "roll_sample_logprob", "roll_policy_loss",
    "roll_policy_loss_workspace_bytes",
    "roll_sample_buffer_create", "roll_sample_buffer_destroy", "roll_sample_buffer_begin",
    "roll_sample_buffer_complete", "roll_sample_buffer_abort", "roll_sample_buffer_resume",
    "roll_sample_buffer_take_batch", "roll_sample_buffer_advance_version", "roll_sample_buffer_version",
    "roll_sample_buffer_outstanding", "roll_sample_buffer_capacity",
    "roll_prof_attn_events", "roll_prof_prefill_events", "roll_prof_attn_timeline", "roll_prof_prefill_timeline", "roll_prof_prefill_units", "roll_prof_kv_read_probe", "roll_prof_event_create", "roll_prof_event_destroy", "roll_prof_event_record",
    "roll_prof_event_elapsed_ms",
]


class RollError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"roll status {status}: {message}")
        self.status = status


class KvConfig(C.Structure):
    _fields_ = [("num_pages", C.c_int32), ("page_size", C.c_int32), ("num_slots", C.c_int32),
                ("max_pages_per_seq", C.c_int32), ("run_pages", C.c_int32)]


class AttnDesc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("page_size", C.c_int32), ("max_pages_per_seq", C.c_int32),
                ("num_pages", C.c_int32), ("out_dtype", C.c_int32), ("softmax_scale", C.c_float),
                ("page_stride", C.c_int64)]


class LossDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("num_seqs", C.c_int32), ("eps_low", C.c_float), ("eps_high", C.c_float),
                ("c", C.c_float)]


LOSS_KINDS = {"ppo": 0, "decoupled_ppo": 1, "tis": 2, "cispo": 3, "topr": 4}


class PrefillDesc(C.Structure):
    _fields_ = [("num_chunks", C.c_int32), ("num_tokens", C.c_int32), ("num_q_heads", C.c_int32),
                ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("page_size", C.c_int32),
                ("max_pages_per_seq", C.c_int32), ("num_pages", C.c_int32), ("num_slots", C.c_int32),
                ("out_dtype", C.c_int32), ("softmax_scale", C.c_float), ("page_stride", C.c_int64)]


class SampleDesc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("vocab", C.c_int32), ("row_stride", C.c_int64),
                ("logits_dtype", C.c_int32), ("policy_version", C.c_int32), ("row_ids", C.c_void_p),
                ("raw_logprob_out", C.c_void_p), ("policy_version_out", C.c_void_p)]


_lib = None


def lib():
    """Load the built library (build it first with ``python -m paper_2510_11345_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: run `python -m paper_2510_11345_amd.build` "
                "(or __graft_entry__.build()) first")
        L = C.CDLL(LIB_PATH)
        L.roll_last_error.restype = C.c_char_p
        L.roll_version.restype = C.c_char_p
        L.roll_decode_attn_workspace_bytes.restype = C.c_size_t
        L.roll_decode_attn_workspace_bytes.argtypes = [C.POINTER(AttnDesc)]
        L.roll_sample_logprob_workspace_bytes.restype = C.c_size_t
        L.roll_sample_logprob_workspace_bytes.argtypes = [C.POINTER(SampleDesc)]
        L.roll_kv_pool_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(KvConfig), C.c_void_p, C.c_void_p]
        L.roll_kv_pool_destroy.argtypes = [C.c_void_p]
        L.roll_kv_alloc.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        L.roll_kv_alloc_batch.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]
        L.roll_kv_release.argtypes = [C.c_void_p, C.c_int32]
        L.roll_kv_commit.argtypes = [C.c_void_p, C.c_void_p]
        L.roll_kv_commit_append.argtypes = [C.c_void_p] * 5 + [C.c_int32, C.c_int32, C.c_int64, C.c_void_p]
        L.roll_kv_free_pages.argtypes = [C.c_void_p]
        L.roll_kv_fused_steps.argtypes = [C.c_void_p]
        L.roll_kv_fused_steps.restype = C.c_int64
        L.roll_kv_seq_len.argtypes = [C.c_void_p, C.c_int32]
        L.roll_kv_slot_pages.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_int32]
        L.roll_kv_append_tokens.argtypes = [C.c_void_p] * 5 + [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p] + \
            [C.c_int32] * 5 + [C.c_int64, C.c_void_p]
        L.roll_decode_attn_workspace_init.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p]
        L.roll_decode_attn_workspace_check.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p]
        L.roll_decode_attn_static.argtypes = [C.c_void_p] * 6 + [C.POINTER(AttnDesc), C.c_void_p]
        L.roll_prof_attn_events.argtypes = [C.c_void_p, C.c_void_p]
        L.roll_prof_prefill_events.argtypes = [C.c_void_p, C.c_void_p]
        L.roll_prof_attn_timeline.argtypes = [C.c_void_p, C.c_size_t]
        L.roll_prof_prefill_timeline.argtypes = [C.c_void_p, C.c_size_t]
        L.roll_prof_prefill_units.argtypes = [C.c_int32]
        L.roll_prof_kv_read_probe.argtypes = [C.c_void_p] * 4 + [C.POINTER(AttnDesc), C.c_void_p, C.c_size_t,
                                              C.POINTER(C.c_int64), C.c_void_p]
        L.roll_decode_attn_ranges.argtypes = [C.POINTER(AttnDesc), C.c_void_p, C.c_int32, C.c_void_p, C.c_int32,
                                              C.POINTER(C.c_int32)]
        L.roll_decode_attn.argtypes = [C.c_void_p] * 6 + [C.POINTER(AttnDesc), C.c_void_p, C.c_size_t, C.c_void_p]
        L.roll_decode_step_attn.argtypes = [C.c_void_p] * 7 + [C.POINTER(AttnDesc), C.c_void_p, C.c_size_t, C.c_void_p]
        L.roll_prefill_attn.argtypes = [C.c_void_p] * 10 + [C.POINTER(PrefillDesc), C.c_void_p]
        L.roll_sample_logprob.argtypes = [C.c_void_p, C.c_float, C.c_float, C.c_uint64, C.c_uint64,
                                          C.c_void_p, C.c_void_p, C.POINTER(SampleDesc), C.c_void_p,
                                          C.c_size_t, C.c_void_p]
        L.roll_policy_loss.argtypes = [C.c_void_p] * 10 + [C.POINTER(LossDesc), C.c_void_p, C.c_size_t, C.c_void_p]
        L.roll_policy_loss_workspace_bytes.restype = C.c_size_t
        L.roll_policy_loss_workspace_bytes.argtypes = [C.POINTER(LossDesc)]
        L.roll_sample_buffer_create.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.c_double]
        L.roll_sample_buffer_destroy.argtypes = [C.c_void_p]
        L.roll_sample_buffer_begin.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        L.roll_sample_buffer_complete.argtypes = [C.c_void_p, C.c_int64, C.c_uint64]
        L.roll_sample_buffer_abort.argtypes = [C.c_void_p, C.c_int64]
        L.roll_sample_buffer_resume.argtypes = [C.c_void_p, C.c_int64, C.POINTER(C.c_int64)]
        L.roll_sample_buffer_take_batch.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.roll_sample_buffer_advance_version.argtypes = [C.c_void_p]
        for f in (L.roll_sample_buffer_version, L.roll_sample_buffer_outstanding, L.roll_sample_buffer_capacity):
            f.argtypes = [C.c_void_p]
            f.restype = C.c_int64
        L.roll_prof_event_create.argtypes = [C.POINTER(C.c_void_p)]
        L.roll_prof_event_destroy.argtypes = [C.c_void_p]
        L.roll_prof_event_record.argtypes = [C.c_void_p, C.c_void_p]
        L.roll_prof_event_elapsed_ms.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_float)]
        _lib = L
    return _lib


def _check(status: int) -> int:
    if status < 0:
        raise RollError(status, lib().roll_last_error().decode())
    return status


def _stream() -> Optional[int]:
    if not torch.cuda.is_available():  # host-only use (allocator logic); GPU calls fail in the library
        return None
    return torch.cuda.current_stream().cuda_stream


def _dev(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("expected a CUDA (ROCm) tensor")
    if not t.is_contiguous():
        raise ValueError("expected a contiguous tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _pool(t: torch.Tensor) -> int:
    """Device pointer of a KV pool: bf16, pages dense inside, any stride between pages."""
    if not t.is_cuda or t.dtype != torch.bfloat16:
        raise ValueError("expected a bf16 CUDA (ROCm) tensor")
    if not t[0].is_contiguous():
        raise ValueError("the pages of a pool must be dense")
    return t.data_ptr()


def page_stride(k_pages: torch.Tensor, v_pages: torch.Tensor) -> int:
    """Elements between consecutive pages of the two pools: 0 for dense pools, the common stride
    for K and V views of one allocation (see `new_kv_pools`)."""
    sk, sv = k_pages.stride(0), v_pages.stride(0)
    if sk != sv:
        raise ValueError("k_pages and v_pages must have the same page stride")
    return 0 if sk == k_pages[0].numel() else sk


def new_kv_pools(num_pages: int, num_kv_heads: int, head_dim: int, page_size: int, device="cuda", fill=None):
    """K and V pools as two views of ONE allocation in which the K block and the V block of a page
    sit side by side (the layout the header recommends).  fill: None (uninitialised) or 0."""
    Hkv, D, P = num_kv_heads, head_dim, page_size
    make = torch.zeros if fill == 0 else torch.empty
    both = make((num_pages, 2, Hkv * P * D), dtype=torch.bfloat16, device=device)
    k = both[:, 0].view(num_pages, Hkv, D // 8, P, 8)
    v = both[:, 1].view(num_pages, Hkv, P // 8, D, 8)
    return k, v


def roll_version() -> str:
    return lib().roll_version().decode()


# ----------------------------------------------------------------------------
# allocator
# ----------------------------------------------------------------------------
class KvPool:
    """Owner of a roll_kv_pool handle.  page_table / seq_lens are device int32 tensors
    (or both None for a host-only pool)."""

    def __init__(self, num_pages: int, page_size: int, num_slots: int, max_pages_per_seq: int,
                 page_table: Optional[torch.Tensor] = None, seq_lens: Optional[torch.Tensor] = None,
                 run_pages: int = 1):
        self.cfg = KvConfig(num_pages, page_size, num_slots, max_pages_per_seq, run_pages)
        self.page_table, self.seq_lens = page_table, seq_lens
        if page_table is not None:
            assert tuple(page_table.shape) == (num_slots, max_pages_per_seq)
            assert tuple(seq_lens.shape) == (num_slots,)
        self._h = C.c_void_p()
        _check(lib().roll_kv_pool_create(C.byref(self._h), C.byref(self.cfg),
                                         _dev(page_table, torch.int32), _dev(seq_lens, torch.int32)))

    def close(self):
        if self._h:
            _check(lib().roll_kv_pool_destroy(self._h))
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def roll_kv_alloc(pool: KvPool, slot: int, n_tokens: int) -> None:
    _check(lib().roll_kv_alloc(pool._h, slot, n_tokens))


def roll_kv_alloc_batch(pool: KvPool, slots, n_tokens) -> None:
    """slots, n_tokens: host int32 numpy arrays of equal length."""
    import numpy as np
    slots = np.ascontiguousarray(slots, dtype=np.int32)
    n_tokens = np.ascontiguousarray(n_tokens, dtype=np.int32)
    assert slots.shape == n_tokens.shape and slots.ndim == 1
    _check(lib().roll_kv_alloc_batch(pool._h, slots.ctypes.data, n_tokens.ctypes.data, len(slots)))


def roll_kv_release(pool: KvPool, slot: int) -> None:
    _check(lib().roll_kv_release(pool._h, slot))


def roll_kv_commit(pool: KvPool) -> None:
    _check(lib().roll_kv_commit(pool._h, _stream()))


def roll_kv_commit_append(pool: KvPool, k_new, v_new, k_pages, v_pages) -> None:
    """Publish the tables and write k_new[slot], v_new[slot] at position seq_len - 1 of every live slot."""
    n, Hkv, D = k_new.shape
    assert n == pool.cfg.num_slots and tuple(v_new.shape) == (n, Hkv, D)
    _check(lib().roll_kv_commit_append(pool._h, _dev(k_new, torch.bfloat16), _dev(v_new, torch.bfloat16),
                                       _pool(k_pages), _pool(v_pages), Hkv, D, page_stride(k_pages, v_pages),
                                       _stream()))


def roll_kv_fused_steps(pool: KvPool) -> int:
    return _check(lib().roll_kv_fused_steps(pool._h))


def roll_kv_free_pages(pool: KvPool) -> int:
    return _check(lib().roll_kv_free_pages(pool._h))


def roll_kv_seq_len(pool: KvPool, slot: int) -> int:
    return _check(lib().roll_kv_seq_len(pool._h, slot))


def roll_kv_slot_pages(pool: KvPool, slot: int) -> list:
    n = _check(lib().roll_kv_slot_pages(pool._h, slot, None, 0))
    buf = (C.c_int32 * max(n, 1))()
    _check(lib().roll_kv_slot_pages(pool._h, slot, buf, n))
    return list(buf[:n])


def roll_kv_append_tokens(k_new, v_new, slots, positions, seq_lens, k_pages, v_pages, page_table,
                          page_size: int) -> None:
    """slots None: token i belongs to slot i; positions None: last token of the slot."""
    n, Hkv, D = k_new.shape
    _check(lib().roll_kv_append_tokens(
        _dev(k_new, torch.bfloat16), _dev(v_new, torch.bfloat16), _dev(slots, torch.int32),
        _dev(positions, torch.int32), _dev(seq_lens, torch.int32), n,
        _pool(k_pages), _pool(v_pages),
        _dev(page_table, torch.int32), page_table.shape[1], k_pages.shape[0], page_size, Hkv, D,
        page_stride(k_pages, v_pages), _stream()))


# ----------------------------------------------------------------------------
# attention
# ----------------------------------------------------------------------------
def attn_desc(q, k_pages, page_table, page_size, out_dtype=torch.bfloat16, softmax_scale=0.0) -> AttnDesc:
    """The page stride is taken from k_pages (the calls check that v_pages has the same)."""
    B, Hq, D = q.shape
    stride = k_pages.stride(0)
    return AttnDesc(B, Hq, k_pages.shape[1], D, page_size, page_table.shape[1], k_pages.shape[0],
                    ROLL_F32 if out_dtype == torch.float32 else ROLL_BF16, softmax_scale,
                    0 if stride == k_pages[0].numel() else stride)


def roll_decode_attn_workspace_bytes(desc: AttnDesc) -> int:
    n = lib().roll_decode_attn_workspace_bytes(C.byref(desc))
    if n == 0:
        raise RollError(-1, lib().roll_last_error().decode())
    return n


def roll_decode_attn_ranges(desc: AttnDesc, seq_lens, workgroups: int = 256):
    """First step of every range roll_decode_attn would cut this batch into (host arithmetic only),
    as an int32 array of num_ranges + 1 entries."""
    import numpy as np
    lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
    if lens.shape != (desc.batch,):
        raise ValueError("seq_lens must hold one length per row")
    n = C.c_int32(0)
    cap = 4 * 256 * 4 + 2
    out = np.zeros(cap, dtype=np.int32)
    _check(lib().roll_decode_attn_ranges(C.byref(desc), lens.ctypes.data, workgroups, out.ctypes.data, cap,
                                         C.byref(n)))
    return out[:n.value + 1].copy()


def roll_decode_attn_workspace_init(workspace: torch.Tensor) -> None:
    _check(lib().roll_decode_attn_workspace_init(_dev(workspace), workspace.numel() * workspace.element_size(),
                                                 _stream()))


def new_attn_workspace(desc: AttnDesc, device="cuda") -> torch.Tensor:
    """Allocate and prepare a workspace for desc."""
    ws = torch.empty(roll_decode_attn_workspace_bytes(desc), dtype=torch.uint8, device=device)
    roll_decode_attn_workspace_init(ws)
    return ws


def roll_decode_attn(q, k_pages, v_pages, page_table, seq_lens, out, desc: AttnDesc,
                     workspace: torch.Tensor) -> None:
    if page_stride(k_pages, v_pages) != desc.page_stride:
        raise ValueError("the pools' page stride differs from the desc's")
    _check(lib().roll_decode_attn(
        _dev(q, torch.bfloat16), _pool(k_pages), _pool(v_pages),
        _dev(page_table, torch.int32), _dev(seq_lens, torch.int32), _dev(out), C.byref(desc),
        _dev(workspace), workspace.numel() * workspace.element_size(), _stream()))


def roll_decode_attn_workspace_check(workspace: torch.Tensor) -> None:
    """Diagnostic (synchronises): raises RollError unless the workspace is prepared, was refused by no
    launch and holds no counters left over from an unfinished one."""
    _check(lib().roll_decode_attn_workspace_check(_dev(workspace), workspace.numel() * workspace.element_size(),
                                                  _stream()))


def roll_decode_attn_static(q, k_pages, v_pages, page_table, seq_lens, out, desc: AttnDesc) -> None:
    """roll_decode_attn on the library's own static scratch (allocates nothing)."""
    if page_stride(k_pages, v_pages) != desc.page_stride:
        raise ValueError("the pools' page stride differs from the desc's")
    _check(lib().roll_decode_attn_static(
        _dev(q, torch.bfloat16), _pool(k_pages), _pool(v_pages),
        _dev(page_table, torch.int32), _dev(seq_lens, torch.int32), _dev(out), C.byref(desc), _stream()))


def roll_decode_step_attn(pool: "KvPool", k_new, v_new, q, k_pages, v_pages, out, desc: AttnDesc,
                          workspace: torch.Tensor) -> None:
    if page_stride(k_pages, v_pages) != desc.page_stride:
        raise ValueError("the pools' page stride differs from the desc's")
    _check(lib().roll_decode_step_attn(
        pool._h, _dev(k_new, torch.bfloat16), _dev(v_new, torch.bfloat16), _dev(q, torch.bfloat16),
        _pool(k_pages), _pool(v_pages), _dev(out), C.byref(desc),
        _dev(workspace), workspace.numel() * workspace.element_size(), _stream()))


def roll_prefill_attn(q, k_new, v_new, chunk_slot, chunk_start, chunk_offset, k_pages, v_pages, page_table,
                      out, page_size: int, softmax_scale: float = 0.0) -> None:
    """Chunked prefill: K/V of the chunk tokens into the pages, then causal attention per token."""
    T, Hq, D = q.shape
    Hkv = k_new.shape[1]
    n_chunks = chunk_slot.shape[0]
    assert tuple(k_new.shape) == (T, Hkv, D) and tuple(v_new.shape) == (T, Hkv, D)
    assert tuple(out.shape) == (T, Hq, D) and chunk_start.shape[0] == n_chunks
    assert chunk_offset.shape[0] == n_chunks + 1
    if out.dtype not in (torch.bfloat16, torch.float32):
        raise TypeError("out must be bfloat16 or float32")
    desc = PrefillDesc(n_chunks, T, Hq, Hkv, D, page_size, page_table.shape[1], k_pages.shape[0],
                       page_table.shape[0], ROLL_BF16 if out.dtype == torch.bfloat16 else ROLL_F32,
                       softmax_scale, page_stride(k_pages, v_pages))
    _check(lib().roll_prefill_attn(
        _dev(q, torch.bfloat16), _dev(k_new, torch.bfloat16), _dev(v_new, torch.bfloat16),
        _dev(chunk_slot, torch.int32), _dev(chunk_start, torch.int32), _dev(chunk_offset, torch.int32),
        _pool(k_pages), _pool(v_pages), _dev(page_table, torch.int32),
        _dev(out), C.byref(desc), _stream()))


# ----------------------------------------------------------------------------
# sampling
# ----------------------------------------------------------------------------
def sample_desc(logits, row_ids=None, raw_logprob_out=None, policy_version: int = 0,
                policy_version_out=None) -> SampleDesc:
    B, V = logits.shape
    dt = ROLL_BF16 if logits.dtype == torch.bfloat16 else ROLL_F32
    if logits.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("logits must be bf16 or fp32")
    if logits.stride(1) != 1:
        raise ValueError("logits rows must be dense")
    return SampleDesc(B, V, logits.stride(0), dt, policy_version, _dev(row_ids, torch.int32),
                      _dev(raw_logprob_out, torch.float32), _dev(policy_version_out, torch.int32))


def roll_sample_logprob_workspace_bytes(desc: SampleDesc) -> int:
    n = lib().roll_sample_logprob_workspace_bytes(C.byref(desc))
    if n == 0:
        raise RollError(-1, lib().roll_last_error().decode())
    return n


def roll_sample_logprob(logits, temperature, top_p, philox_seed, step, tokens_out, logprob_out,
                        desc: SampleDesc, workspace: Optional[torch.Tensor] = None) -> None:
    if not logits.is_cuda:
        raise ValueError("expected a CUDA (ROCm) tensor")
    _check(lib().roll_sample_logprob(
        logits.data_ptr(), temperature, top_p, philox_seed, step, _dev(tokens_out, torch.int32),
        _dev(logprob_out, torch.float32), C.byref(desc), _dev(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream()))


# ----------------------------------------------------------------------------
# consumer of the log-probs
# ----------------------------------------------------------------------------
_loss_workspaces = {}


def roll_policy_loss_workspace_bytes(num_seqs: int) -> int:
    desc = LossDesc(0, num_seqs, 0.2, 0.2, 5.0)
    return lib().roll_policy_loss_workspace_bytes(C.byref(desc))


def roll_policy_loss(kind, logp_theta, logp_old, logp_prox, signal, seq_offsets, value_out, grad_out,
                     is_weight_out, seq_mean_out, batch_mean_out, eps_low=0.2, eps_high=0.2, c=5.0,
                     workspace: Optional[torch.Tensor] = None) -> None:
    """workspace None: one buffer per device is kept and reused (calls are then ordered on the
    current stream by the caller, as any two calls that share a workspace must be)."""
    desc = LossDesc(LOSS_KINDS[kind], seq_offsets.numel() - 1, eps_low, eps_high, c)
    if workspace is None:
        key = logp_theta.device.index
        if key not in _loss_workspaces:
            _loss_workspaces[key] = torch.empty(lib().roll_policy_loss_workspace_bytes(C.byref(desc)),
                                                dtype=torch.uint8, device=logp_theta.device)
        workspace = _loss_workspaces[key]
    _check(lib().roll_policy_loss(
        _dev(logp_theta, torch.float32), _dev(logp_old, torch.float32), _dev(logp_prox, torch.float32),
        _dev(signal, torch.float32), _dev(seq_offsets, torch.int64), _dev(value_out, torch.float32),
        _dev(grad_out, torch.float32), _dev(is_weight_out, torch.float32), _dev(seq_mean_out, torch.float32),
        _dev(batch_mean_out, torch.float32), C.byref(desc), _dev(workspace),
        workspace.numel() * workspace.element_size(), _stream()))


# ----------------------------------------------------------------------------
# SampleBuffer (host only)
# ----------------------------------------------------------------------------
class SampleBuffer:
    def __init__(self, batch_size: int, alpha: float):
        self.batch_size = batch_size
        self._h = C.c_void_p()
        _check(lib().roll_sample_buffer_create(C.byref(self._h), batch_size, alpha))

    def begin(self):
        """(ticket, init_version), or None when the buffer is at capacity."""
        t, v = C.c_int64(), C.c_int64()
        st = lib().roll_sample_buffer_begin(self._h, C.byref(t), C.byref(v))
        if st == -8:
            return None
        _check(st)
        return t.value, v.value

    def complete(self, ticket: int, payload: int = 0):
        _check(lib().roll_sample_buffer_complete(self._h, ticket, payload))

    def abort(self, ticket: int):
        _check(lib().roll_sample_buffer_abort(self._h, ticket))

    def resume(self, ticket: int) -> int:
        v = C.c_int64()
        _check(lib().roll_sample_buffer_resume(self._h, ticket, C.byref(v)))
        return v.value

    def take_batch(self):
        """List of (ticket, init_version, payload), or None when the trainer has to wait."""
        n = self.batch_size
        t, v, p = (C.c_int64 * n)(), (C.c_int64 * n)(), (C.c_uint64 * n)()
        st = lib().roll_sample_buffer_take_batch(self._h, t, v, p)
        if st == -9:
            return None
        _check(st)
        return list(zip(t, v, p))

    def advance_version(self) -> bool:
        st = lib().roll_sample_buffer_advance_version(self._h)
        if st == -9:
            return False
        _check(st)
        return True

    version = property(lambda self: lib().roll_sample_buffer_version(self._h))
    outstanding = property(lambda self: lib().roll_sample_buffer_outstanding(self._h))
    capacity = property(lambda self: lib().roll_sample_buffer_capacity(self._h))

    def __del__(self):
        try:
            if self._h:
                lib().roll_sample_buffer_destroy(self._h)
        except Exception:
            pass


# ----------------------------------------------------------------------------
# profiling events
# ----------------------------------------------------------------------------
def roll_prof_attn_events(begin: Optional["ProfEvent"], end: Optional["ProfEvent"]) -> None:
    """The calling thread's next attention launches record these two events around the kernel;
    (None, None) switches that off."""
    _check(lib().roll_prof_attn_events(None if begin is None else begin.handle, None if end is None else end.handle))


def roll_prof_prefill_events(begin: Optional["ProfEvent"], end: Optional["ProfEvent"]) -> None:
    """The same for roll_prefill_attn: the events bracket its attention kernel."""
    _check(lib().roll_prof_prefill_events(None if begin is None else begin.handle, None if end is None else end.handle))


def roll_prof_attn_timeline(buffer: Optional[torch.Tensor]) -> None:
    """Per-wave timestamps of the next attention launches into `buffer` (a library built with
    `python -m paper_2510_11345_amd.build --timeline` only); None switches it off."""
    _check(lib().roll_prof_attn_timeline(_dev(buffer), 0 if buffer is None else buffer.numel() * buffer.element_size()))


def roll_prof_prefill_units(units: int) -> None:
    """Units (span of query tokens x query head) per prefill workgroup for head groups of up to 8:
    1 .. 8, or 0 for the choice per launch (the default).  Applies to the calling thread."""
    _check(lib().roll_prof_prefill_units(units))


def roll_prof_prefill_timeline(buffer: Optional[torch.Tensor]) -> None:
    """Per-workgroup timestamps of the next prefill attention launches into `buffer` (int64,
    8 words per workgroup; a library built with `python -m paper_2510_11345_amd.build --timeline`
    only); None switches it off."""
    _check(lib().roll_prof_prefill_timeline(_dev(buffer), 0 if buffer is None else buffer.numel() * buffer.element_size()))


def roll_prof_kv_read_probe(k_pages, v_pages, page_table, seq_lens, desc: AttnDesc, sink: torch.Tensor) -> int:
    """Enqueue the plain read of the batch's paged KV bytes; returns the bytes it reads per page."""
    per_page = C.c_int64()
    _check(lib().roll_prof_kv_read_probe(_pool(k_pages), _pool(v_pages), _dev(page_table, torch.int32),
                                         _dev(seq_lens, torch.int32), C.byref(desc), _dev(sink),
                                         sink.numel() * sink.element_size(), C.byref(per_page), _stream()))
    return per_page.value


class ProfEvent:
    def __init__(self):
        self._h = C.c_void_p()
        _check(lib().roll_prof_event_create(C.byref(self._h)))

    @property
    def handle(self):
        return self._h

    def record(self):
        _check(lib().roll_prof_event_record(self._h, _stream()))

    def elapsed_ms(self, end: "ProfEvent") -> float:
        ms = C.c_float()
        _check(lib().roll_prof_event_elapsed_ms(self._h, end._h, C.byref(ms)))
        return ms.value

    def __del__(self):
        try:
            if self._h:
                lib().roll_prof_event_destroy(self._h)
        except Exception:
            pass
