"""fp64 CPU oracle of the rollout decode step (test infrastructure only).

Thin ctypes wrapper around ``roll_oracle.c``.  Nothing here is imported by
the GPU package; only tests, the smoke check and the benchmark's CPU
baseline use it.  Arrays are numpy; bf16 tensors travel as ``uint16`` bit
patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "roll_oracle.c")
# ROLL_ORACLE_SANITIZE=1 (set by tests/test_sanitizers.py for a child process that preloads the
# sanitizer runtime) selects a second build of the same source with AddressSanitizer and
# UndefinedBehaviorSanitizer, so that the pins also prove the oracle reads and writes in bounds.
SANITIZE = os.environ.get("ROLL_ORACLE_SANITIZE", "") == "1"
_LIB = os.path.join(_HERE, "libroll_oracle_san.so" if SANITIZE else "libroll_oracle.so")

BF16, F32 = 0, 1
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over independent rows / heads only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        opt = (["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                "-fno-sanitize-recover=all"] if SANITIZE else ["-O2"])
        cmd = ["gcc", *opt, "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t)) if a is not None else None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.oracle_uniform.restype = C.c_double
        L.oracle_uniform.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32]
        L.oracle_bf16_to_double.restype = C.c_double
        L.oracle_bf16_to_double.argtypes = [C.c_uint16]
        L.oracle_k_index.restype = C.c_int64
        L.oracle_v_index.restype = C.c_int64
        for f in (L.oracle_k_index, L.oracle_v_index):
            f.argtypes = [C.c_int64] + [C.c_int] * 6
        L.oracle_k_slot.restype = C.c_int
        L.oracle_k_slot.argtypes = [C.c_int, C.c_int]
        L.oracle_top_p_cut.restype = C.c_double
        L.oracle_top_p_cut.argtypes = [C.POINTER(C.c_double), C.c_int, C.c_double, C.c_double]
        L.oracle_decode_attn.restype = C.c_int
        L.oracle_prefill_attn.restype = C.c_int
        L.oracle_sample_logprob.restype = C.c_int
        _lib = L
    return _lib


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*[int(v) & 0xFFFFFFFF for v in ctr])
    k = (C.c_uint32 * 2)(*[int(v) & 0xFFFFFFFF for v in key])
    o = (C.c_uint32 * 4)()
    lib().oracle_philox4x32_10(c, k, o)
    return [int(v) for v in o]


def uniform(seed, step, row_id, i):
    return float(lib().oracle_uniform(int(seed), int(step), int(row_id), int(i)))


def k_slot(t, P):
    return int(lib().oracle_k_slot(t, P))


def k_index(page, h, t, d, Hkv, D, P):
    return int(lib().oracle_k_index(page, h, t, d, Hkv, D, P))


def v_index(page, h, t, d, Hkv, D, P):
    return int(lib().oracle_v_index(page, h, t, d, Hkv, D, P))


def kv_store(k_pages, v_pages, page, t, k_tok, v_tok, Hkv, D, P):
    """Write one token's K/V ([Hkv, D] uint16 each) at position t of a page."""
    k_tok = np.ascontiguousarray(k_tok, dtype=np.uint16)
    v_tok = np.ascontiguousarray(v_tok, dtype=np.uint16)
    lib().oracle_kv_store(_p(k_pages, C.c_uint16), _p(v_pages, C.c_uint16), C.c_int64(page),
                          C.c_int(t), _p(k_tok, C.c_uint16), _p(v_tok, C.c_uint16),
                          C.c_int(Hkv), C.c_int(D), C.c_int(P))


def attn_range(q, k_pages, v_pages, page_table, b, h, j0, j1, Hq, Hkv, D, P, scale=None):
    """(m, l, acc[D]) of one (row, head) over KV positions [j0, j1)."""
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    m, l = C.c_double(), C.c_double()
    acc = np.zeros(D, dtype=np.float64)
    page_table = np.ascontiguousarray(page_table, dtype=np.int32)
    lib().oracle_attn_range(_p(q, C.c_uint16), _p(k_pages, C.c_uint16), _p(v_pages, C.c_uint16),
                            _p(page_table, C.c_int32), C.c_int(b), C.c_int(h), C.c_int(j0),
                            C.c_int(j1), C.c_int(Hq), C.c_int(Hkv), C.c_int(D), C.c_int(P),
                            C.c_int(page_table.shape[1]), C.c_double(scale),
                            C.byref(m), C.byref(l), _p(acc, C.c_double))
    return m.value, l.value, acc


def decode_attn(q, k_pages, v_pages, page_table, seq_lens, Hq, Hkv, D, P, scale=None,
                rows=None, n_threads=0, return_threads=False):
    """out[B, Hq, D] fp64.  q uint16 [B, Hq, D]; pools uint16; tables int32."""
    for a in (q, k_pages, v_pages):
        assert a.dtype == np.uint16 and a.flags.c_contiguous
    page_table = np.ascontiguousarray(page_table, dtype=np.int32)
    seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
    B = seq_lens.shape[0]
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    out = np.zeros((B, Hq, D), dtype=np.float64)
    r = None if rows is None else np.ascontiguousarray(rows, dtype=np.int32)
    used = lib().oracle_decode_attn(
        _p(q, C.c_uint16), _p(k_pages, C.c_uint16), _p(v_pages, C.c_uint16),
        _p(page_table, C.c_int32), _p(seq_lens, C.c_int32), _p(out, C.c_double),
        C.c_int(B), C.c_int(Hq), C.c_int(Hkv), C.c_int(D), C.c_int(P),
        C.c_int(page_table.shape[1]), C.c_double(scale), _p(r, C.c_int32),
        C.c_int(0 if r is None else len(r)), C.c_int(n_threads))
    return (out, used) if return_threads else out


def prefill_attn(q, k_new, v_new, chunk_slot, chunk_start, chunk_offset, k_pages, v_pages, page_table,
                 Hq, Hkv, D, P, scale=None, n_threads=0):
    """Chunked prefill: writes the chunk tokens' K/V into k_pages / v_pages IN PLACE (uint16 pools)
    and returns out[T, Hq, D] fp64, token (c, j) attending over positions 0 .. chunk_start[c] + j
    of slot chunk_slot[c].  q uint16 [T, Hq, D]; k_new, v_new uint16 [T, Hkv, D]."""
    for a in (q, k_new, v_new, k_pages, v_pages):
        assert a.dtype == np.uint16 and a.flags.c_contiguous
    cs = np.ascontiguousarray(chunk_slot, dtype=np.int32)
    st = np.ascontiguousarray(chunk_start, dtype=np.int32)
    off = np.ascontiguousarray(chunk_offset, dtype=np.int32)
    page_table = np.ascontiguousarray(page_table, dtype=np.int32)
    n_chunks, T = len(cs), int(off[-1])
    assert len(st) == n_chunks and len(off) == n_chunks + 1 and q.shape[0] == T
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    out = np.zeros((T, Hq, D), dtype=np.float64)
    lib().oracle_prefill_attn(
        _p(q, C.c_uint16), _p(k_new, C.c_uint16), _p(v_new, C.c_uint16), _p(cs, C.c_int32),
        _p(st, C.c_int32), _p(off, C.c_int32), C.c_int(n_chunks), _p(k_pages, C.c_uint16),
        _p(v_pages, C.c_uint16), _p(page_table, C.c_int32), _p(out, C.c_double), C.c_int(Hq),
        C.c_int(Hkv), C.c_int(D), C.c_int(P), C.c_int(page_table.shape[1]), C.c_double(scale),
        C.c_int(n_threads))
    return out


def _logits_args(logits):
    assert logits.ndim == 2 and logits.strides[1] == logits.itemsize
    if logits.dtype == np.uint16:
        dt = BF16
    elif logits.dtype == np.float32:
        dt = F32
    else:
        raise TypeError("logits must be uint16 (bf16 bits) or float32")
    return dt, logits.shape[0], logits.shape[1], logits.strides[0] // logits.itemsize


def sample_logprob(logits, temperature, top_p, seed, step, row_ids=None, band=1e-5,
                   n_threads=0):
    """Returns dict(tokens, logprob, raw_logprob, gap, kept, x_cut, x_cut_minus, x_cut_plus, threads)."""
    dt, B, V, stride = _logits_args(logits)
    tokens = np.zeros(B, np.int32)
    kept = np.zeros(B, np.int32)
    lp, gap, xc, xm, xp, raw = (np.zeros(B, np.float64) for _ in range(6))
    rid = None if row_ids is None else np.ascontiguousarray(row_ids, dtype=np.int32)
    used = lib().oracle_sample_logprob(
        C.c_void_p(logits.ctypes.data), C.c_int(dt), C.c_int(B), C.c_int(V), C.c_int64(stride),
        C.c_double(float(np.float32(temperature))), C.c_double(float(np.float32(top_p))),
        C.c_uint64(seed), C.c_uint64(step), _p(rid, C.c_int32), C.c_double(band),
        _p(tokens, C.c_int32), _p(lp, C.c_double), _p(gap, C.c_double), _p(kept, C.c_int32),
        _p(xc, C.c_double), _p(xm, C.c_double), _p(xp, C.c_double), _p(raw, C.c_double),
        C.c_int(n_threads))
    return dict(tokens=tokens, logprob=lp, raw_logprob=raw, gap=gap, kept=kept, x_cut=xc,
                x_cut_minus=xm, x_cut_plus=xp, threads=used)


def top_p_cut(x, temperature, top_p):
    x = np.ascontiguousarray(x, dtype=np.float64)
    return float(lib().oracle_top_p_cut(_p(x, C.c_double), C.c_int(len(x)),
                                        C.c_double(temperature), C.c_double(top_p)))


def row_detail(row, temperature, top_p, seed, step, row_id=0):
    """(perturbed[V], kept[V]) of one row."""
    row = np.ascontiguousarray(row)
    dt = BF16 if row.dtype == np.uint16 else F32
    V = row.shape[0]
    pert = np.zeros(V, np.float64)
    kept = np.zeros(V, np.uint8)
    lib().oracle_row_detail(C.c_void_p(row.ctypes.data), C.c_int(dt), C.c_int(V),
                            C.c_double(temperature), C.c_double(top_p), C.c_uint64(seed),
                            C.c_uint64(step), C.c_uint32(row_id), _p(pert, C.c_double),
                            _p(kept, C.c_uint8))
    return pert, kept.astype(bool)


def sample_counts(row, temperature, top_p, seed, step0, n_draws, row_id=0):
    row = np.ascontiguousarray(row)
    dt = BF16 if row.dtype == np.uint16 else F32
    V = row.shape[0]
    counts = np.zeros(V, np.int64)
    lib().oracle_sample_counts(C.c_void_p(row.ctypes.data), C.c_int(dt), C.c_int(V),
                               C.c_double(temperature), C.c_double(top_p), C.c_uint64(seed),
                               C.c_uint64(step0), C.c_int64(n_draws), C.c_uint32(row_id),
                               _p(counts, C.c_int64))
    return counts


LOSS_KINDS = {"ppo": 0, "decoupled_ppo": 1, "tis": 2, "cispo": 3, "topr": 4}


def policy_loss(kind, logp_theta, logp_old, logp_prox, signal, offsets, eps_lo=0.2, eps_hi=0.2, c=5.0):
    """Off-policy objectives over ragged responses.  Arrays are float32 [T]; offsets int64 [n_seq+1].
    Returns dict(value, grad, is_weight [T], seq_mean [n_seq], batch_mean)."""
    lt = np.ascontiguousarray(logp_theta, np.float32)
    lo = np.ascontiguousarray(logp_old, np.float32)
    lp = None if logp_prox is None else np.ascontiguousarray(logp_prox, np.float32)
    R = np.ascontiguousarray(signal, np.float32)
    off = np.ascontiguousarray(offsets, np.int64)
    T, n = len(lt), len(off) - 1
    value, grad, w = (np.zeros(T, np.float64) for _ in range(3))
    seq_mean = np.zeros(n, np.float64)
    bm = C.c_double()
    lib().oracle_policy_loss(C.c_int(LOSS_KINDS[kind]), _p(lt, C.c_float), _p(lo, C.c_float), _p(lp, C.c_float),
                             _p(R, C.c_float), _p(off, C.c_int64), C.c_int(n), C.c_double(eps_lo),
                             C.c_double(eps_hi), C.c_double(c), _p(value, C.c_double), _p(grad, C.c_double),
                             _p(w, C.c_double), _p(seq_mean, C.c_double), C.byref(bm))
    return dict(value=value, grad=grad, is_weight=w, seq_mean=seq_mean, batch_mean=bm.value)
