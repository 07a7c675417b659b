"""ctypes binding of the rollout_attn C ABI (include/rollout_attn.h).  Argument marshalling only: every
step of the decode path runs in the library's kernels.  There is no fallback: if the shared library is
missing the import of a symbol raises."""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "librollout_attn.so")
_lib = None

RA_OK, RA_ERR_INVALID_ARG, RA_ERR_UNSUPPORTED, RA_ERR_WORKSPACE_TOO_SMALL, RA_ERR_OUT_OF_RANGE, RA_ERR_DEVICE = range(6)
RA_KV_BF16, RA_KV_FP8_E4M3 = 0, 1
RA_FLAG_VALIDATE, RA_FLAG_NO_PREFIX_SHARING, RA_FLAG_REUSE_SCHEDULE = 1, 2, 4
_STATUS_NAMES = ["RA_OK", "RA_ERR_INVALID_ARG", "RA_ERR_UNSUPPORTED", "RA_ERR_WORKSPACE_TOO_SMALL",
                 "RA_ERR_OUT_OF_RANGE", "RA_ERR_DEVICE"]


class RolloutAttnError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("%s: %s" % (_STATUS_NAMES[status] if 0 <= status < 6 else status, message))
        self.status = status


class ra_problem(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32),
        ("page_size", ctypes.c_int32), ("num_pages", ctypes.c_int32), ("max_pages_per_seq", ctypes.c_int32),
        ("q", ctypes.c_void_p), ("k_pool", ctypes.c_void_p), ("v_pool", ctypes.c_void_p),
        ("kv_stride_page", ctypes.c_int64), ("kv_stride_head", ctypes.c_int64), ("kv_stride_token", ctypes.c_int64),
        ("kv_dtype", ctypes.c_int32),
        ("k_scale", ctypes.c_void_p), ("v_scale", ctypes.c_void_p),
        ("block_table", ctypes.c_void_p), ("seq_lens", ctypes.c_void_p),
        ("num_groups", ctypes.c_int32),
        ("seq_group", ctypes.c_void_p), ("prefix_page_offsets", ctypes.c_void_p), ("prefix_pages", ctypes.c_void_p),
        ("softmax_scale", ctypes.c_float),
        ("out", ctypes.c_void_p), ("lse", ctypes.c_void_p),
        ("flags", ctypes.c_uint32),
    ]


class ra_prefill(ctypes.Structure):
    _fields_ = [
        ("num_prompts", ctypes.c_int32), ("total_tokens", ctypes.c_int32), ("max_prompt_len", ctypes.c_int32),
        ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32),
        ("q", ctypes.c_void_p), ("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("cu_seqlens", ctypes.c_void_p),
        ("softmax_scale", ctypes.c_float),
        ("out", ctypes.c_void_p), ("lse", ctypes.c_void_p),
        ("k_pool", ctypes.c_void_p), ("v_pool", ctypes.c_void_p),
        ("page_size", ctypes.c_int32), ("num_pages", ctypes.c_int32),
        ("kv_stride_page", ctypes.c_int64), ("kv_stride_head", ctypes.c_int64), ("kv_stride_token", ctypes.c_int64),
        ("kv_dtype", ctypes.c_int32),
        ("k_scale", ctypes.c_void_p), ("v_scale", ctypes.c_void_p),
        ("page_offsets", ctypes.c_void_p), ("pages", ctypes.c_void_p),
    ]


def library_path():
    return _LIB_PATH


def load_library():
    """Loads librollout_attn.so (built by paper_2507_01663_amd/build.py).  Raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("%s is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or python paper_2507_01663_amd/build.py) first" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    P = ctypes.POINTER
    lib.rollout_attn_abi_version.restype = ctypes.c_uint32
    lib.rollout_attn_abi_version.argtypes = []
    lib.rollout_attn_create.restype = ctypes.c_int
    lib.rollout_attn_create.argtypes = [P(ctypes.c_void_p), ctypes.c_int]
    lib.rollout_attn_destroy.restype = None
    lib.rollout_attn_destroy.argtypes = [ctypes.c_void_p]
    lib.rollout_attn_last_error.restype = ctypes.c_char_p
    lib.rollout_attn_last_error.argtypes = [ctypes.c_void_p]
    lib.rollout_attn_check_problem.restype = ctypes.c_int
    lib.rollout_attn_check_problem.argtypes = [P(ra_problem), ctypes.c_char_p, ctypes.c_size_t]
    lib.rollout_attn_workspace_size.restype = ctypes.c_int
    lib.rollout_attn_workspace_size.argtypes = [ctypes.c_void_p, P(ra_problem), P(ctypes.c_size_t)]
    lib.rollout_attn_decode.restype = ctypes.c_int
    lib.rollout_attn_decode.argtypes = [ctypes.c_void_p, P(ra_problem), ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.rollout_attn_decode_static.restype = ctypes.c_int
    lib.rollout_attn_decode_static.argtypes = [ctypes.c_void_p, P(ra_problem), ctypes.c_void_p]
    lib.rollout_attn_debug_gather.restype = ctypes.c_int
    lib.rollout_attn_debug_gather.argtypes = [ctypes.c_void_p, P(ra_problem), ctypes.c_int32, ctypes.c_int32,
                                              ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    lib.rollout_attn_debug_schedule.restype = ctypes.c_int
    lib.rollout_attn_debug_schedule.argtypes = [ctypes.c_void_p, P(ra_problem), ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                                P(ra_schedule_info)]
    lib.rollout_attn_append.restype = ctypes.c_int
    lib.rollout_attn_append.argtypes = [ctypes.c_void_p, P(ra_problem), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    lib.rollout_attn_check_prefill.restype = ctypes.c_int
    lib.rollout_attn_check_prefill.argtypes = [P(ra_prefill), ctypes.c_char_p, ctypes.c_size_t]
    lib.rollout_attn_prefill.restype = ctypes.c_int
    lib.rollout_attn_prefill.argtypes = [ctypes.c_void_p, P(ra_prefill), ctypes.c_void_p]
    lib.rollout_attn_balance.restype = ctypes.c_int
    lib.rollout_attn_balance.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
    lib.rollout_attn_wave_count.restype = ctypes.c_int
    lib.rollout_attn_wave_count.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, P(ctypes.c_int32)]
    lib.rollout_attn_set_wave_weights.restype = ctypes.c_int
    lib.rollout_attn_set_wave_weights.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32]
    lib.rollout_attn_debug_stream.restype = ctypes.c_int
    lib.rollout_attn_debug_stream.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int32,
                                              ctypes.c_int32, ctypes.c_void_p, P(ctypes.c_size_t)]
    lib.rollout_attn_debug_stream_tail.restype = ctypes.c_int
    lib.rollout_attn_debug_stream_tail.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int32,
                                                   ctypes.c_int32, ctypes.c_void_p, P(ctypes.c_size_t)]
    lib.rollout_attn_set_timing.restype = ctypes.c_int
    lib.rollout_attn_set_timing.argtypes = [ctypes.c_void_p, ctypes.c_int]
    lib.rollout_attn_get_timing.restype = ctypes.c_int
    lib.rollout_attn_get_timing.argtypes = [ctypes.c_void_p, P(ctypes.c_float)]
    _lib = lib
    return lib


# ---- the C entry points, same names, status codes turned into exceptions ------------------------------

def rollout_attn_abi_version():
    return int(load_library().rollout_attn_abi_version())


def rollout_attn_last_error(ctx):
    s = load_library().rollout_attn_last_error(ctx)
    return s.decode() if s else ""


def _check(status, ctx):
    if status != RA_OK:
        raise RolloutAttnError(status, rollout_attn_last_error(ctx))


def rollout_attn_create(device_ordinal=0):
    ctx = ctypes.c_void_p()
    _check(load_library().rollout_attn_create(ctypes.byref(ctx), int(device_ordinal)), None)
    return ctx


def rollout_attn_destroy(ctx):
    load_library().rollout_attn_destroy(ctx)


def rollout_attn_check_problem(problem):
    """Returns (status, message) of the host-side argument check."""
    buf = ctypes.create_string_buffer(512)
    st = load_library().rollout_attn_check_problem(ctypes.byref(problem) if problem is not None else None, buf, 512)
    return int(st), buf.value.decode()


def rollout_attn_workspace_size(ctx, problem):
    n = ctypes.c_size_t()
    _check(load_library().rollout_attn_workspace_size(ctx, ctypes.byref(problem), ctypes.byref(n)), ctx)
    return int(n.value)


def rollout_attn_decode(ctx, problem, workspace_ptr, workspace_bytes, hip_stream=None):
    _check(load_library().rollout_attn_decode(ctx, ctypes.byref(problem), workspace_ptr, workspace_bytes, hip_stream), ctx)


def rollout_attn_decode_static(ctx, problem, hip_stream=None):
    _check(load_library().rollout_attn_decode_static(ctx, ctypes.byref(problem), hip_stream), ctx)


def rollout_attn_debug_gather(ctx, problem, b, kv_head, k_out_ptr, v_out_ptr, capacity_tokens, hip_stream=None):
    _check(load_library().rollout_attn_debug_gather(ctx, ctypes.byref(problem), b, kv_head, k_out_ptr, v_out_ptr,
                                                    capacity_tokens, hip_stream), ctx)


def rollout_attn_debug_schedule(ctx, problem, workspace_ptr, workspace_bytes, hip_stream=None):
    info = ra_schedule_info()
    _check(load_library().rollout_attn_debug_schedule(ctx, ctypes.byref(problem), workspace_ptr, workspace_bytes, hip_stream,
                                                      ctypes.byref(info)), ctx)
    return info


def rollout_attn_append(ctx, problem, k_new_ptr, v_new_ptr, hip_stream=None):
    _check(load_library().rollout_attn_append(ctx, ctypes.byref(problem), k_new_ptr, v_new_ptr, hip_stream), ctx)


def rollout_attn_check_prefill(prefill):
    """Returns (status, message) of the host-side argument check of a prefill."""
    buf = ctypes.create_string_buffer(512)
    st = load_library().rollout_attn_check_prefill(ctypes.byref(prefill) if prefill is not None else None, buf, 512)
    return int(st), buf.value.decode()


def rollout_attn_prefill(ctx, prefill, hip_stream=None):
    _check(load_library().rollout_attn_prefill(ctx, ctypes.byref(prefill), hip_stream), ctx)


def rollout_attn_balance(weights, k, equal_count=False):
    """(part, part_sums) as numpy arrays; weights: non-negative integers."""
    import numpy as np
    w = np.ascontiguousarray(weights, dtype=np.int64)
    part = np.empty(w.size, dtype=np.int32)
    sums = np.empty(max(int(k), 0), dtype=np.int64)
    _check(load_library().rollout_attn_balance(w.ctypes.data, w.size, int(k), int(bool(equal_count)), part.ctypes.data,
                                               sums.ctypes.data), None)
    return part, sums


def rollout_attn_wave_count(ctx, kv_dtype=RA_KV_BF16, head_dim=128):
    n = ctypes.c_int32()
    _check(load_library().rollout_attn_wave_count(ctx, kv_dtype, head_dim, ctypes.byref(n)), ctx)
    return int(n.value)


def rollout_attn_set_wave_weights(ctx, weights, kv_dtype=RA_KV_BF16, head_dim=128):
    """weights: per mille of the mean, one per attention workgroup of the launch shape (host integers)."""
    import numpy as np
    w = np.ascontiguousarray(weights, dtype=np.int32)
    _check(load_library().rollout_attn_set_wave_weights(ctx, kv_dtype, head_dim, w.ctypes.data, w.size), ctx)


def rollout_attn_debug_stream(ctx, buf_ptr, buf_bytes, granule_bytes, scattered, entries_per_wave, hip_stream=None):
    """Enqueues the streaming probe; returns the bytes the launch reads."""
    n = ctypes.c_size_t()
    _check(load_library().rollout_attn_debug_stream(ctx, buf_ptr, buf_bytes, granule_bytes, int(scattered) & 3, entries_per_wave,
                                                    hip_stream, ctypes.byref(n)), ctx)
    return int(n.value)


def rollout_attn_debug_stream_tail(ctx, buf_ptr, buf_bytes, entries_per_wave, static_entries, chunk_entries, hip_stream=None):
    """Enqueues the streaming probe with a ticketed tail; returns the bytes the launch reads."""
    n = ctypes.c_size_t()
    _check(load_library().rollout_attn_debug_stream_tail(ctx, buf_ptr, buf_bytes, entries_per_wave, static_entries, chunk_entries,
                                                         hip_stream, ctypes.byref(n)), ctx)
    return int(n.value)


def rollout_attn_set_timing(ctx, enable):
    _check(load_library().rollout_attn_set_timing(ctx, int(bool(enable))), ctx)


def rollout_attn_get_timing(ctx):
    """(schedule_ms, attention_ms, merge_ms) of the most recent timed decode call."""
    ms = (ctypes.c_float * 3)()
    _check(load_library().rollout_attn_get_timing(ctx, ms), ctx)
    return tuple(float(x) for x in ms)


# ---- helpers over torch tensors (device memory and streams only) --------------------------------------

def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def problem_from_tensors(q, k_pool, v_pool, block_table, seq_lens, out, lse, softmax_scale, k_scale=None, v_scale=None,
                         seq_group=None, prefix_page_offsets=None, prefix_pages=None, flags=0):
    """Fills a ra_problem from device tensors: q/out bf16 [B,Hq,D]; pools [num_pages,Hkv,page,D] bf16 or uint8
    (any strides with D contiguous); block_table int32 [B,max_pages]; seq_lens int32 [B]; lse float32 [B,Hq]."""
    import torch
    assert q.is_contiguous() and out.is_contiguous() and lse.is_contiguous()
    assert block_table.is_contiguous() and seq_lens.is_contiguous()
    assert q.dtype == torch.bfloat16 and out.dtype == torch.bfloat16 and lse.dtype == torch.float32
    assert block_table.dtype == torch.int32 and seq_lens.dtype == torch.int32
    assert k_pool.stride() == v_pool.stride() and k_pool.stride(3) == 1
    p = ra_problem()
    p.B, p.Hq, p.D = q.shape
    p.num_pages, p.Hkv, p.page_size, _ = k_pool.shape
    p.max_pages_per_seq = block_table.shape[1]
    p.q, p.k_pool, p.v_pool = _ptr(q), _ptr(k_pool), _ptr(v_pool)
    p.kv_stride_page, p.kv_stride_head, p.kv_stride_token = k_pool.stride(0), k_pool.stride(1), k_pool.stride(2)
    p.kv_dtype = RA_KV_FP8_E4M3 if k_pool.element_size() == 1 else RA_KV_BF16
    p.k_scale, p.v_scale = _ptr(k_scale), _ptr(v_scale)
    p.block_table, p.seq_lens = _ptr(block_table), _ptr(seq_lens)
    if seq_group is not None:
        assert seq_group.dtype == torch.int32 and prefix_page_offsets.dtype == torch.int32 and prefix_pages.dtype == torch.int32
        p.num_groups = prefix_page_offsets.numel() - 1
        p.seq_group, p.prefix_page_offsets, p.prefix_pages = _ptr(seq_group), _ptr(prefix_page_offsets), _ptr(prefix_pages)
    p.softmax_scale = float(softmax_scale)
    p.out, p.lse = _ptr(out), _ptr(lse)
    p.flags = flags
    return p


def prefill_from_tensors(q, k, v, cu_seqlens, max_prompt_len, out, lse, softmax_scale, k_pool=None, v_pool=None, k_scale=None,
                         v_scale=None, page_offsets=None, pages=None):
    """Fills a ra_prefill from device tensors: q/out bf16 [T,Hq,D]; k/v bf16 [T,Hkv,D]; cu_seqlens int32 [n+1];
    lse float32 [T,Hq]; optionally the pools [num_pages,Hkv,page,D] (bf16 or uint8) and the prompts' page lists."""
    import torch
    for t in (q, k, v, out, lse, cu_seqlens):
        assert t.is_contiguous()
    assert q.dtype == k.dtype == v.dtype == out.dtype == torch.bfloat16 and lse.dtype == torch.float32
    assert cu_seqlens.dtype == torch.int32 and k.shape == v.shape and q.shape == out.shape
    p = ra_prefill()
    p.total_tokens, p.Hq, p.D = q.shape
    p.Hkv = k.shape[1]
    p.num_prompts = cu_seqlens.numel() - 1
    p.max_prompt_len = int(max_prompt_len)
    p.q, p.k, p.v, p.cu_seqlens = _ptr(q), _ptr(k), _ptr(v), _ptr(cu_seqlens)
    p.softmax_scale = float(softmax_scale)
    p.out, p.lse = _ptr(out), _ptr(lse)
    if k_pool is not None:
        assert k_pool.stride() == v_pool.stride() and k_pool.stride(3) == 1
        assert page_offsets.dtype == torch.int32 and pages.dtype == torch.int32
        p.k_pool, p.v_pool = _ptr(k_pool), _ptr(v_pool)
        p.num_pages, _, p.page_size, _ = k_pool.shape
        p.kv_stride_page, p.kv_stride_head, p.kv_stride_token = k_pool.stride(0), k_pool.stride(1), k_pool.stride(2)
        p.kv_dtype = RA_KV_FP8_E4M3 if k_pool.element_size() == 1 else RA_KV_BF16
        p.k_scale, p.v_scale = _ptr(k_scale), _ptr(v_scale)
        p.page_offsets, p.pages = _ptr(page_offsets), _ptr(pages)
    return p


class ra_schedule_info(ctypes.Structure):
    _fields_ = [("header_offset", ctypes.c_int64), ("work_list_offset", ctypes.c_int64), ("merge_desc_offset", ctypes.c_int64),
                ("waves", ctypes.c_int32), ("segments_per_chunk", ctypes.c_int32)]


class Decoder:
    """A context plus a cached workspace tensor on one device.  The workspace grows when a larger problem arrives;
    the tensors it outgrew stay alive until close(), because work already enqueued (or a HIP graph captured earlier)
    may still use them.  A captured graph and a schedule that RA_FLAG_REUSE_SCHEDULE reuses are tied to the workspace
    they were made with: after the workspace has grown, capture or schedule again."""

    def __init__(self, device_ordinal=0):
        self.device_ordinal = device_ordinal
        self.ctx = rollout_attn_create(device_ordinal)
        self._ws = None
        self._retired = []

    def close(self):
        if self.ctx is not None:
            import torch
            torch.cuda.synchronize(self.device_ordinal)      # nothing enqueued may outlive the buffers
            rollout_attn_destroy(self.ctx)
            self.ctx = None
            self._ws = None
            self._retired = []

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def workspace(self, problem):
        import torch
        need = rollout_attn_workspace_size(self.ctx, problem)
        if self._ws is None or self._ws.numel() < need:
            if self._ws is not None:
                self._retired.append(self._ws)
            self._ws = torch.empty(need, dtype=torch.uint8, device="cuda:%d" % self.device_ordinal)
        return self._ws

    def decode(self, problem, stream=None):
        """Enqueues one decode step on the given (or the current) torch stream."""
        import torch
        ws = self.workspace(problem)
        s = stream if stream is not None else torch.cuda.current_stream(self.device_ordinal)
        rollout_attn_decode(self.ctx, problem, ctypes.c_void_p(ws.data_ptr()), ws.numel(), ctypes.c_void_p(s.cuda_stream))

    def decode_static(self, problem, stream=None):
        """The same step on the library's built-in workspace (no allocation anywhere)."""
        import torch
        s = stream if stream is not None else torch.cuda.current_stream(self.device_ordinal)
        rollout_attn_decode_static(self.ctx, problem, ctypes.c_void_p(s.cuda_stream))

    def schedule(self, problem, stream=None):
        """Runs only the schedule; returns (ra_schedule_info, the workspace tensor it was written to)."""
        import torch
        ws = self.workspace(problem)
        s = stream if stream is not None else torch.cuda.current_stream(self.device_ordinal)
        info = rollout_attn_debug_schedule(self.ctx, problem, ctypes.c_void_p(ws.data_ptr()), ws.numel(), ctypes.c_void_p(s.cuda_stream))
        return info, ws

    def append(self, problem, k_new, v_new, stream=None):
        """Enqueues the KV append of one token per sequence (k_new, v_new: bf16 tensors [B, Hkv, D])."""
        import torch
        s = stream if stream is not None else torch.cuda.current_stream(self.device_ordinal)
        rollout_attn_append(self.ctx, problem, _ptr(k_new), _ptr(v_new), ctypes.c_void_p(s.cuda_stream))

    def prefill(self, prefill, stream=None):
        """Enqueues the prompts' causal attention (and the cache write, if the ra_prefill names pools)."""
        import torch
        s = stream if stream is not None else torch.cuda.current_stream(self.device_ordinal)
        rollout_attn_prefill(self.ctx, prefill, ctypes.c_void_p(s.cuda_stream))

    def debug_gather(self, problem, b, kv_head, k_out, v_out, stream=None):
        import torch
        s = stream if stream is not None else torch.cuda.current_stream(self.device_ordinal)
        rollout_attn_debug_gather(self.ctx, problem, b, kv_head, _ptr(k_out), _ptr(v_out), k_out.shape[0],
                                  ctypes.c_void_p(s.cuda_stream))
