"""fp64 CPU oracle for paged decode attention.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the product path never does.  It shares no code with the HIP
library and does not import it.  The arithmetic lives in
``rollout_attn_oracle.c`` (plain C, fp64, two-pass softmax in logical token
order); this module only marshals numpy arrays into that C code.

The paper motivates the computation (memory-bound auto-regressive rollout,
Sec. 2.1.1; groups of responses to one prompt, Sec. 7.1; highly variable
response lengths, Sec. 7.4) but prints no formula for it; the definition
used is textbook scaled-dot-product attention with grouped query heads and a
paged cache, as written out at the top of the C file.  The same C file holds
the oracle of the KV append (``append`` below) and of the prompt prefill and
its cache write (``prefill``, ``prefill_write``); ``oracle/balance.py`` is the
oracle of the token-balanced dispatch.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


class _CProblem(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32),
        ("page_size", ctypes.c_int32), ("num_pages", ctypes.c_int32), ("max_pages_per_seq", ctypes.c_int32),
        ("kv_dtype", ctypes.c_int32),
        ("q", ctypes.c_void_p), ("k_pool", ctypes.c_void_p), ("v_pool", ctypes.c_void_p),
        ("stride_page", ctypes.c_int64), ("stride_head", ctypes.c_int64), ("stride_token", ctypes.c_int64),
        ("k_scale", ctypes.c_void_p), ("v_scale", ctypes.c_void_p),
        ("block_table", ctypes.c_void_p), ("seq_lens", ctypes.c_void_p),
        ("softmax_scale", ctypes.c_float),
    ]


def _lib():
    global _LIB
    if _LIB is None:
        path = _build.build()
        lib = ctypes.CDLL(path)
        lib.oracle_decode.restype = ctypes.c_int
        lib.oracle_decode.argtypes = [ctypes.POINTER(_CProblem), ctypes.c_void_p, ctypes.c_int64,
                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        lib.oracle_probs.restype = ctypes.c_int
        lib.oracle_probs.argtypes = [ctypes.POINTER(_CProblem), ctypes.c_int, ctypes.c_int,
                                     ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_gather.restype = ctypes.c_int
        lib.oracle_gather.argtypes = [ctypes.POINTER(_CProblem), ctypes.c_int, ctypes.c_int,
                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_e4m3_decode.restype = ctypes.c_double
        lib.oracle_e4m3_decode.argtypes = [ctypes.c_uint8]
        lib.oracle_threads.restype = ctypes.c_int
        lib.oracle_e4m3_encode.restype = ctypes.c_uint8
        lib.oracle_e4m3_encode.argtypes = [ctypes.c_float]
        lib.oracle_prefill.restype = ctypes.c_int
        lib.oracle_prefill.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int,
                                       ctypes.c_int, ctypes.c_int, ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        lib.oracle_prefill_write.restype = ctypes.c_int
        lib.oracle_prefill_write.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                             ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                             ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_append.restype = ctypes.c_int
        lib.oracle_append.argtypes = [ctypes.POINTER(_CProblem), ctypes.c_void_p, ctypes.c_void_p]
        _LIB = lib
    return _LIB


class _Marshalled:
    """Keeps the contiguous numpy views alive next to the C struct."""

    def __init__(self, p):
        fp8 = p.kv_dtype == "fp8_e4m3"
        pool_dt = np.uint8 if fp8 else np.uint16
        self.q = np.ascontiguousarray(p.q, dtype=np.uint16)
        self.k = np.ascontiguousarray(p.k_pool, dtype=pool_dt)
        self.v = np.ascontiguousarray(p.v_pool, dtype=pool_dt)
        self.bt = np.ascontiguousarray(p.block_table, dtype=np.int32)
        self.sl = np.ascontiguousarray(p.seq_lens, dtype=np.int32)
        self.ks = np.ascontiguousarray(p.k_scale, dtype=np.float32) if fp8 else None
        self.vs = np.ascontiguousarray(p.v_scale, dtype=np.float32) if fp8 else None
        B, Hq, D = self.q.shape
        num_pages, Hkv, page, D2 = self.k.shape
        assert D2 == D and self.v.shape == self.k.shape
        assert self.bt.shape[0] == B and self.sl.shape == (B,)
        c = _CProblem()
        c.B, c.Hq, c.Hkv, c.D = B, Hq, Hkv, D
        c.page_size, c.num_pages, c.max_pages_per_seq = page, num_pages, self.bt.shape[1]
        c.kv_dtype = 1 if fp8 else 0
        c.q = self.q.ctypes.data
        c.k_pool, c.v_pool = self.k.ctypes.data, self.v.ctypes.data
        c.stride_page, c.stride_head, c.stride_token = Hkv * page * D, page * D, D
        c.k_scale = self.ks.ctypes.data if fp8 else None
        c.v_scale = self.vs.ctypes.data if fp8 else None
        c.block_table, c.seq_lens = self.bt.ctypes.data, self.sl.ctypes.data
        c.softmax_scale = float(np.float32(p.softmax_scale))
        self.c = c
        self.B, self.Hq, self.Hkv, self.D = B, Hq, Hkv, D


def _raise(rc):
    if rc:
        raise ValueError({1: "bad problem or row id", 2: "page id or length out of range",
                          3: "out of memory"}.get(rc, "oracle status %d" % rc))


def decode(p, rows=None, nthreads=0):
    """Attention of every (b, h) row, or of the listed rows (row id = b*Hq + h).

    ``p`` is any object with the fields of ``workload.Problem``: q (bf16 bits,
    uint16 [B,Hq,D]), k_pool / v_pool ([num_pages,Hkv,page,D] uint16 bf16 bits
    or uint8 e4m3 codes), kv_dtype, k_scale / v_scale, block_table, seq_lens,
    softmax_scale.  Returns (out float64 [n, D], lse float64 [n]) with n = B*Hq
    or len(rows); with rows=None, out is reshaped to [B,Hq,D] and lse to [B,Hq].
    """
    m = _Marshalled(p)
    if rows is None:
        n, rptr = m.B * m.Hq, None
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        n, rptr = rows.size, rows.ctypes.data
    out = np.empty((n, m.D), dtype=np.float64)
    lse = np.empty((n,), dtype=np.float64)
    _raise(_lib().oracle_decode(ctypes.byref(m.c), rptr, n, out.ctypes.data, lse.ctypes.data, nthreads))
    if rows is None:
        return out.reshape(m.B, m.Hq, m.D), lse.reshape(m.B, m.Hq)
    return out, lse


def probs(p, b, h):
    """Softmax weights p_t (t < L_b) of one row, with its output and lse."""
    m = _Marshalled(p)
    L = int(m.sl[b])
    pr = np.empty((max(L, 1),), dtype=np.float64)
    out = np.empty((m.D,), dtype=np.float64)
    lse = np.empty((1,), dtype=np.float64)
    _raise(_lib().oracle_probs(ctypes.byref(m.c), b, h, pr.ctypes.data, out.ctypes.data, lse.ctypes.data))
    return pr[:L], out, float(lse[0])


def gather(p, b, kv):
    """Stored K and V elements of sequence b, KV head kv, in logical token
    order: two arrays [L_b, D] of the pool's raw element type, plus the physical
    page id of every token."""
    m = _Marshalled(p)
    L = int(m.sl[b])
    k = np.empty((L, m.D), dtype=m.k.dtype)
    v = np.empty((L, m.D), dtype=m.k.dtype)
    pages = np.empty((L,), dtype=np.int32)
    _raise(_lib().oracle_gather(ctypes.byref(m.c), b, kv, k.ctypes.data, v.ctypes.data, pages.ctypes.data))
    return k, v, pages


def e4m3_decode_table():
    """The 256 values of the OCP E4M3 format, by code."""
    lib = _lib()
    return np.array([lib.oracle_e4m3_decode(c) for c in range(256)], dtype=np.float64)


def merge_partials(outs, lses):
    """Combine attention results over disjoint key sets into the result over
    their union: with weights w_i = exp(lse_i - M), M = max_i lse_i,
    out = sum_i w_i out_i / sum_i w_i and lse = M + ln sum_i w_i.
    outs: [n, D] float64, lses: [n] float64 (-inf marks an empty set)."""
    outs = np.asarray(outs, dtype=np.float64)
    lses = np.asarray(lses, dtype=np.float64)
    M = np.max(lses)
    if not np.isfinite(M):
        return np.zeros(outs.shape[1:], dtype=np.float64), -np.inf
    w = np.exp(lses - M)
    return (w[:, None] * outs).sum(axis=0) / w.sum(), float(M + np.log(w.sum()))


def threads():
    return int(_lib().oracle_threads())


def e4m3_encode(x):
    """Nearest OCP E4M3 code (ties to even, saturating at 448, NaN -> 0x7F) of every binary32 value in x."""
    lib = _lib()
    x = np.asarray(x, dtype=np.float32)
    return np.array([lib.oracle_e4m3_encode(float(v)) for v in x.ravel()], dtype=np.uint8).reshape(x.shape)


def append(p, k_new, v_new):
    """Appends one token per sequence at position seq_lens[b] (paged write; e4m3 pools quantise on write and
    maintain the per-(page, head) scales as described in the C file).  ``p.k_pool``, ``p.v_pool`` (and
    ``p.k_scale``, ``p.v_scale``) must be C-contiguous numpy arrays of the pool's type; they are modified in
    place.  ``k_new``, ``v_new``: bf16 bits, uint16 [B, Hkv, D].  ``p.seq_lens`` is not changed.  Returns the
    number of sequences skipped because their length or page id is out of range."""
    fp8 = p.kv_dtype == "fp8_e4m3"
    for a, dt in ((p.k_pool, np.uint8 if fp8 else np.uint16), (p.v_pool, np.uint8 if fp8 else np.uint16)):
        assert a.dtype == dt and a.flags["C_CONTIGUOUS"] and a.flags["WRITEABLE"]
    if fp8:
        for a in (p.k_scale, p.v_scale):
            assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"] and a.flags["WRITEABLE"]
    m = _Marshalled(p)  # its views alias the arrays checked above
    assert m.k.ctypes.data == p.k_pool.ctypes.data and m.v.ctypes.data == p.v_pool.ctypes.data
    kn = np.ascontiguousarray(k_new, dtype=np.uint16)
    vn = np.ascontiguousarray(v_new, dtype=np.uint16)
    assert kn.shape == (m.B, m.Hkv, m.D) and vn.shape == kn.shape
    return int(_lib().oracle_append(ctypes.byref(m.c), kn.ctypes.data, vn.ctypes.data))


def prefill(q, k, v, cu_seqlens, softmax_scale, nthreads=0):
    """Causal attention of packed prompts over themselves (the arithmetic of the prefill that fills a group's
    shared pages).  q: bf16 bits uint16 [T, Hq, D]; k, v: [T, Hkv, D]; cu_seqlens: int32 [groups + 1].
    Returns (out float64 [T, Hq, D], lse float64 [T, Hq])."""
    q = np.ascontiguousarray(q, dtype=np.uint16)
    k = np.ascontiguousarray(k, dtype=np.uint16)
    v = np.ascontiguousarray(v, dtype=np.uint16)
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (T, Hkv, D) and v.shape == k.shape and cu[0] == 0 and cu[-1] == T
    out = np.empty((T, Hq, D), dtype=np.float64)
    lse = np.empty((T, Hq), dtype=np.float64)
    _raise(_lib().oracle_prefill(q.ctypes.data, k.ctypes.data, v.ctypes.data, cu.ctypes.data, cu.size - 1, Hq, Hkv, D,
                                 float(np.float32(softmax_scale)), out.ctypes.data, lse.ctypes.data, nthreads))
    return out, lse


def prefill_write(k, v, cu_seqlens, page_offsets, pages, k_pool, v_pool, k_scale=None, v_scale=None):
    """Cache write of the prompt prefill (see the C file): the prompts' K and V rows (bf16 bits, uint16
    [T, Hkv, D]) go into the pages listed per prompt.  ``k_pool``, ``v_pool``: C-contiguous
    [num_pages, Hkv, page, D], uint16 (bit patterns are copied) or uint8 (e4m3 codes, one scale per (page, head)
    written to ``k_scale``, ``v_scale``: float32 [num_pages, Hkv]); all modified in place, everything that
    receives no token is left as it was."""
    k = np.ascontiguousarray(k, dtype=np.uint16)
    v = np.ascontiguousarray(v, dtype=np.uint16)
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    po = np.ascontiguousarray(page_offsets, dtype=np.int32)
    pg = np.ascontiguousarray(pages, dtype=np.int32)
    fp8 = k_pool.dtype == np.uint8
    for a in (k_pool, v_pool):
        assert a.dtype == (np.uint8 if fp8 else np.uint16) and a.flags["C_CONTIGUOUS"] and a.flags["WRITEABLE"]
    num_pages, Hkv, page, D = k_pool.shape
    assert v_pool.shape == k_pool.shape and k.shape[1:] == (Hkv, D) and v.shape == k.shape
    assert po.size == cu.size and (pg.size == 0 or po[-1] <= pg.size)
    if fp8:
        for a in (k_scale, v_scale):
            assert a.dtype == np.float32 and a.shape == (num_pages, Hkv) and a.flags["C_CONTIGUOUS"] and a.flags["WRITEABLE"]
    _raise(_lib().oracle_prefill_write(k.ctypes.data, v.ctypes.data, cu.ctypes.data, cu.size - 1, Hkv, D, page, po.ctypes.data,
                                       pg.ctypes.data if pg.size else None, num_pages, 1 if fp8 else 0, k_pool.ctypes.data,
                                       v_pool.ctypes.data, k_scale.ctypes.data if fp8 else None, v_scale.ctypes.data if fp8 else None))
