"""Seeded synthetic decode-attention workloads shaped like GRPO rollout batches.

This module only *makes inputs*: lengths, page tables, pools of random bf16
(or e4m3-encoded) values, queries.  It holds none of the attention arithmetic
and imports neither the HIP library nor the oracle; both are fed the same
arrays from here.

Why these shapes.  The paper measures GRPO on a math dataset with Qwen2.5
checkpoints (Sec. 7.1); neither is available, and attention cost depends only
on head shapes and the structure of the lengths, so the batches below stand
in: N responses share one prompt (GRPO groups, Sec. 7.1), response lengths
vary widely (Sec. 7.4), and the head shapes are those of the public 7B / 32B /
72B model cards.  No dataset item is reproduced.
"""
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
import math
import os

import numpy as np

PAGE = 16
BF16_NAN = 0x7FC0
E4M3_NAN = 0x7F

# name -> shape.  "resp" names the response-length recipe (see response_lengths()).
CONFIGS = {
    # B=4, one group of 4; total KV lengths {17,64,100,256} of which the first 16 are the prompt.
    "tiny": dict(id=0, Hq=4, Hkv=2, D=64, groups=1, R=4, prompt=16, resp="tiny"),
    # 7B-shaped GRPO batch: 32 prompts x 8 responses, prompt 512, responses U[0,3584].
    "grpo7b": dict(id=1, Hq=28, Hkv=4, D=128, groups=32, R=8, prompt=512, resp="uniform", resp_max=3584),
    # 32B-shaped long tail: 64 x 8, prompt 1024, lognormal(median 2048, sigma 0.8) capped at 16384.
    "tail32b": dict(id=2, Hq=40, Hkv=8, D=128, groups=64, R=8, prompt=1024, resp="lognormal",
                    resp_median=2048, resp_sigma=0.8, resp_max=16384),
    # 72B-shaped streaming: 16 x 16, prompt 2048, responses up to 30720, 64 consecutive decode steps.
    "stream72b": dict(id=4, Hq=64, Hkv=8, D=128, groups=16, R=16, prompt=2048, resp="stream",
                      resp_max=30720, p_finish=0.02, steps=64),
    # A batch of the 7B shape without structure, for comparison with "grpo7b" in benchmarks: 256 sequences of
    # 2304 tokens (the GRPO batch's mean), no shared prompts, so every sequence is a group of its own.
    "regular7b": dict(id=21, Hq=28, Hkv=4, D=128, groups=256, R=1, prompt=0, resp="fixed", resp_len=2304),
    # Reduced shapes for element-by-element parity (the oracle finishes them in seconds):
    # several KV tiles per sequence, ragged tails, empty responses, more than one group.
    "mid7b": dict(id=11, Hq=28, Hkv=4, D=128, groups=3, R=8, prompt=80, resp="uniform", resp_max=700),
    "mid32b": dict(id=12, Hq=40, Hkv=8, D=128, groups=2, R=8, prompt=48, resp="lognormal",
                   resp_median=200, resp_sigma=0.8, resp_max=1500),
    "mid72b": dict(id=14, Hq=64, Hkv=8, D=128, groups=2, R=16, prompt=64, resp="stream",
                   resp_max=900, p_finish=0.02, steps=8),
    "midd64": dict(id=15, Hq=8, Hkv=2, D=64, groups=3, R=4, prompt=32, resp="uniform", resp_max=300),
}


@dataclass
class Problem:
    name: str
    B: int
    Hq: int
    Hkv: int
    D: int
    num_pages: int
    max_pages_per_seq: int
    kv_dtype: str                      # "bf16" | "fp8_e4m3"
    q: np.ndarray                      # uint16 bf16 bits [B, Hq, D]
    k_pool: np.ndarray                 # uint16 / uint8 [num_pages, Hkv, PAGE, D]
    v_pool: np.ndarray
    k_scale: np.ndarray                # float32 [num_pages, Hkv] or None
    v_scale: np.ndarray
    block_table: np.ndarray            # int32 [B, max_pages_per_seq], -1 past the last page
    seq_lens: np.ndarray               # int32 [B] total KV tokens (prompt + response)
    num_groups: int
    seq_group: np.ndarray              # int32 [B]
    prefix_page_offsets: np.ndarray    # int32 [num_groups + 1]
    prefix_pages: np.ndarray           # int32 page ids shared by the group
    softmax_scale: np.float32
    page_size: int = PAGE
    meta: dict = field(default_factory=dict)

    @property
    def elem_bytes(self):
        return 1 if self.kv_dtype == "fp8_e4m3" else 2

    def shared_tokens(self):
        """Tokens of each group's shared (whole-page) prefix, per group."""
        return (np.diff(self.prefix_page_offsets) * self.page_size).astype(np.int64)

    def algorithmic_bytes(self, share_prefix=True):
        """Bytes the method itself must move in one decode step: every distinct
        KV token once (shared prompt pages once per group), fp8 scales of the
        touched pages, q in, out and lse out, the touched table entries and the
        lengths.  Page over-fetch and split-KV partials are not counted."""
        e = self.elem_bytes
        per_tok = 2 * self.Hkv * self.D * e
        L = self.seq_lens.astype(np.int64)
        sh = self.shared_tokens()[self.seq_group] if self.num_groups else np.zeros_like(L)
        sh = np.minimum(sh, L)
        if share_prefix and self.num_groups:
            members = np.bincount(self.seq_group, minlength=self.num_groups)
            kv_tok = int((self.shared_tokens() * (members > 0)).sum() + (L - sh).sum())
        else:
            kv_tok = int(L.sum())
        total = kv_tok * per_tok
        if e == 1:
            total += (kv_tok // self.page_size) * 2 * 4 * self.Hkv
        total += 2 * self.B * self.Hq * self.D * 2 + 4 * self.B * self.Hq
        total += 4 * int(((L + self.page_size - 1) // self.page_size).sum()) + 4 * self.B
        return int(total)

    def kv_tokens(self):
        return int(self.seq_lens.astype(np.int64).sum())


# ----------------------------------------------------------------------------
# random values
# ----------------------------------------------------------------------------

def f32_to_bf16_bits(x):
    """Round-to-nearest-even truncation of float32 to its upper 16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


_CHUNK = 1 << 22


def normal_bf16(n, seed, tensor_id):
    """n values ~ N(0,1) rounded to bf16 (bits).  Chunked so that the result
    depends only on (seed, tensor_id, n), not on the number of threads."""
    out = np.empty(n, dtype=np.uint16)
    nchunks = (n + _CHUNK - 1) // _CHUNK

    def fill(c):
        lo, hi = c * _CHUNK, min(n, (c + 1) * _CHUNK)
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, tensor_id, c])))
        out[lo:hi] = f32_to_bf16_bits(rng.standard_normal(hi - lo, dtype=np.float32))

    workers = min(16, len(os.sched_getaffinity(0)), max(1, nchunks))
    if workers > 1:
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(fill, range(nchunks)))
    else:
        for c in range(nchunks):
            fill(c)
    return out


_BASE_ELEMS = (1 << 27) - 24      # not a multiple of a page tile: repeats never line up with pages


def _fill_tiled(total, seed, tensor_id):
    """total bf16 values; beyond _BASE_ELEMS the first block repeats (throughput
    does not depend on the values, and the period is chosen so that no two
    pages hold the same bytes at the same offsets)."""
    if total <= _BASE_ELEMS:
        return normal_bf16(total, seed, tensor_id)
    base = normal_bf16(_BASE_ELEMS, seed, tensor_id)
    out = np.empty(total, dtype=np.uint16)
    for lo in range(0, total, _BASE_ELEMS):
        hi = min(total, lo + _BASE_ELEMS)
        out[lo:hi] = base[: hi - lo]
    return out


def e4m3_encode(y):
    """Nearest OCP E4M3 code (ties to even, saturating at +-448) of float32 y."""
    y = np.asarray(y, dtype=np.float32)
    sign = np.signbit(y)
    a = np.minimum(np.abs(y).astype(np.float64), 448.0)
    _, ex = np.frexp(a)                       # a = m * 2**ex, m in [0.5, 1)
    e = np.maximum(ex - 1, -6)                # binade exponent, clamped to the subnormal range
    step = np.ldexp(1.0, e - 3)
    v = np.minimum(np.rint(a / step) * step, 448.0)     # rint rounds half to even
    _, ex2 = np.frexp(v)
    e2 = np.maximum(ex2 - 1, -6)
    is_sub = v < 2.0 ** -6
    mant = np.where(is_sub, v / 2.0 ** -9, (v / np.ldexp(1.0, e2) - 1.0) * 8.0)
    expo = np.where(is_sub, 0, e2 + 7)
    code = (expo.astype(np.int64) << 3) | np.rint(mant).astype(np.int64)
    code = np.where(v == 0, 0, code)
    return (code | (sign.astype(np.int64) << 7)).astype(np.uint8)


_FP8_BASE_TILES = 16381


def _quantise_tiles(vals_bf16_bits):
    """[n, PAGE*D] bf16 bits -> (uint8 codes, float32 scale[n]); scale =
    absmax/448 in fp32 (1 when the tile is all zero), codes = nearest e4m3 of
    value/scale (fp32 divide)."""
    x = bf16_bits_to_f32(vals_bf16_bits)
    amax = np.abs(x).max(axis=1).astype(np.float32)
    scale = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    return e4m3_encode(x / scale[:, None]), scale


def make_pool(num_pages, Hkv, D, kv_dtype, seed, tensor_id):
    """One pool [num_pages, Hkv, PAGE, D] (+ scales for fp8)."""
    tile = PAGE * D
    ntiles = num_pages * Hkv
    if kv_dtype == "bf16":
        return _fill_tiled(ntiles * tile, seed, tensor_id).reshape(num_pages, Hkv, PAGE, D), None
    nb = min(ntiles, _FP8_BASE_TILES)
    codes, scale = _quantise_tiles(normal_bf16(nb * tile, seed, tensor_id).reshape(nb, tile))
    if nb < ntiles:
        idx = np.arange(ntiles) % nb
        codes, scale = codes[idx], scale[idx]
    return codes.reshape(num_pages, Hkv, PAGE, D), scale.reshape(num_pages, Hkv).copy()


# ----------------------------------------------------------------------------
# lengths
# ----------------------------------------------------------------------------

def _rng(seed, cfg_id, step, what):
    return np.random.default_rng([seed, cfg_id, step, what])


def response_lengths(cfg, seed, step=0):
    """Response length of every sequence at the given decode step."""
    B = cfg["groups"] * cfg["R"]
    kind = cfg["resp"]
    if kind == "tiny":
        return np.array([1, 48, 84, 240], dtype=np.int64)
    if kind == "fixed":
        return np.full(B, cfg["resp_len"], dtype=np.int64)
    if kind == "uniform":
        return _rng(seed, cfg["id"], 0, 1).integers(0, cfg["resp_max"] + 1, size=B)
    if kind == "lognormal":
        z = _rng(seed, cfg["id"], 0, 1).standard_normal(B)
        r = np.rint(np.exp(math.log(cfg["resp_median"]) + cfg["resp_sigma"] * z))
        return np.minimum(r, cfg["resp_max"]).astype(np.int64)
    if kind == "stream":
        # Start uniform; every step each live sequence grows by one token; it
        # finishes with probability p_finish (or at the cap) and its slot is
        # refilled by a new member of the same group with an empty response.
        r = _rng(seed, cfg["id"], 0, 1).integers(0, cfg["resp_max"] + 1, size=B)
        for s in range(1, step + 1):
            fin = (_rng(seed, cfg["id"], s, 2).random(B) < cfg["p_finish"]) | (r >= cfg["resp_max"])
            r = np.where(fin, 0, r + 1)
        return r
    raise ValueError(kind)


# ----------------------------------------------------------------------------
# problems
# ----------------------------------------------------------------------------

def build_problem(name, Hq, Hkv, D, prompt_lens, R, resp_lens, kv_dtype="bf16", seed=0, cfg_id=99, step=0,
                  slack=1.25, poison=True, pool=None, num_pages=None, softmax_scale=None, make_values=True):
    """Lay out groups of R sequences (members contiguous: b = g*R + r) over a
    randomly permuted page pool.  The whole pages of each prompt are stored
    once and appear at the head of every member's block-table row."""
    prompt_lens = np.asarray(prompt_lens, dtype=np.int64)
    resp_lens = np.asarray(resp_lens, dtype=np.int64)
    ngroups = prompt_lens.size
    B = ngroups * R
    assert resp_lens.size == B
    seq_group = np.repeat(np.arange(ngroups, dtype=np.int32), R)
    L = prompt_lens[seq_group] + resp_lens
    npages_seq = (L + PAGE - 1) // PAGE
    shared_pages = prompt_lens // PAGE                       # whole pages only
    own_pages = npages_seq - shared_pages[seq_group]
    needed = int(shared_pages.sum() + own_pages.sum())
    if num_pages is None:
        num_pages = max(needed + 1, int(math.ceil(slack * needed)))
    assert needed <= num_pages
    phys = _rng(seed, cfg_id, step, 3).permutation(num_pages)[:needed].astype(np.int32)

    max_pages = max(1, int(npages_seq.max()))
    block_table = np.full((B, max_pages), -1, dtype=np.int32)
    prefix_page_offsets = np.zeros(ngroups + 1, dtype=np.int32)
    prefix_page_offsets[1:] = np.cumsum(shared_pages)
    prefix_pages = np.empty(int(shared_pages.sum()), dtype=np.int32)
    cur = 0
    for g in range(ngroups):
        ns = int(shared_pages[g])
        sh = phys[cur:cur + ns]
        cur += ns
        prefix_pages[prefix_page_offsets[g]:prefix_page_offsets[g + 1]] = sh
        for r in range(R):
            b = g * R + r
            no = int(own_pages[b])
            block_table[b, :ns] = sh
            block_table[b, ns:ns + no] = phys[cur:cur + no]
            cur += no
    assert cur == needed

    if softmax_scale is None:
        softmax_scale = np.float32(1.0 / math.sqrt(D))
    k_scale = v_scale = None
    if pool is not None:
        k_pool, v_pool, k_scale, v_scale = pool
        assert k_pool.shape == (num_pages, Hkv, PAGE, D)
    elif make_values:
        k_pool, k_scale = make_pool(num_pages, Hkv, D, kv_dtype, seed, 100 + cfg_id * 8 + 0)
        v_pool, v_scale = make_pool(num_pages, Hkv, D, kv_dtype, seed, 100 + cfg_id * 8 + 1)
    else:
        k_pool = v_pool = None
    if poison and k_pool is not None:
        nan = E4M3_NAN if kv_dtype == "fp8_e4m3" else BF16_NAN
        used = np.zeros(num_pages, dtype=bool)
        used[phys] = True
        for pl in (k_pool, v_pool):
            pl[~used] = nan
        # slots past the end of each sequence's last page
        tail = L % PAGE
        for b in np.nonzero(tail)[0]:
            last = block_table[b, npages_seq[b] - 1]
            k_pool[last, :, tail[b]:, :] = nan
            v_pool[last, :, tail[b]:, :] = nan
    q = normal_bf16(B * Hq * D, seed, 100 + cfg_id * 8 + 2 + 8 * 1000 * step).reshape(B, Hq, D) if make_values else None
    return Problem(name=name, B=B, Hq=Hq, Hkv=Hkv, D=D, num_pages=num_pages, max_pages_per_seq=max_pages,
                   kv_dtype=kv_dtype, q=q, k_pool=k_pool, v_pool=v_pool, k_scale=k_scale, v_scale=v_scale,
                   block_table=block_table, seq_lens=L.astype(np.int32), num_groups=ngroups, seq_group=seq_group,
                   prefix_page_offsets=prefix_page_offsets, prefix_pages=prefix_pages,
                   softmax_scale=np.float32(softmax_scale),
                   meta=dict(seed=seed, step=step, prompt_lens=prompt_lens, resp_lens=resp_lens, needed_pages=needed))


def make_problem(config, seed=0, step=0, kv_dtype="bf16", pool=None, num_pages=None, make_values=True):
    """One decode step of a named configuration.

    For the streaming configurations the pool is static across steps: pass the
    (k_pool, v_pool, k_scale, v_scale) of step 0 and its num_pages back in;
    the lengths advance and the block table is re-drawn from (seed, step)."""
    cfg = CONFIGS[config]
    resp = response_lengths(cfg, seed, step)
    prompts = np.full(cfg["groups"], cfg["prompt"], dtype=np.int64)
    stream = cfg["resp"] == "stream"
    if stream and num_pages is None:
        # capacity for every step of the run
        worst = 0
        for s in range(cfg["steps"]):
            Ls = cfg["prompt"] + response_lengths(cfg, seed, s)
            worst = max(worst, int(((Ls + PAGE - 1) // PAGE - cfg["prompt"] // PAGE).sum()))
        num_pages = int(math.ceil(1.25 * (worst + cfg["groups"] * (cfg["prompt"] // PAGE))))
    name = config if kv_dtype == "bf16" else config + "_fp8"
    return build_problem(name, cfg["Hq"], cfg["Hkv"], cfg["D"], prompts, cfg["R"], resp, kv_dtype=kv_dtype,
                         seed=seed, cfg_id=cfg["id"], step=step, poison=not stream, pool=pool,
                         num_pages=num_pages, make_values=make_values)


# ----------------------------------------------------------------------------
# prompt prefill
# ----------------------------------------------------------------------------

@dataclass
class PrefillBatch:
    """Packed prompts for the prefill step: token t of the batch is row t of q
    ([T, Hq, D]) and of k, v ([T, Hkv, D]), all bf16 bit patterns; prompt g is
    rows cu_seqlens[g] .. cu_seqlens[g+1]; its pages are
    pages[page_offsets[g] .. page_offsets[g+1]] of a pool of num_pages."""
    name: str
    Hq: int
    Hkv: int
    D: int
    cu_seqlens: np.ndarray
    q: np.ndarray
    k: np.ndarray
    v: np.ndarray
    softmax_scale: np.float32
    num_pages: int
    page_offsets: np.ndarray
    pages: np.ndarray

    @property
    def lens(self):
        return np.diff(self.cu_seqlens).astype(np.int64)

    def causal_pairs(self):
        """(query, key) pairs of the causal mask, over all prompts."""
        n = self.lens
        return int((n * (n + 1) // 2).sum())

    def flops(self):
        """Multiply-adds of the two products, counted as two operations each."""
        return 4 * self.D * self.Hq * self.causal_pairs()


def build_prefill(name, Hq, Hkv, D, prompt_lens, seed=0, cfg_id=99, slack=1.25):
    """Prompts of the given lengths with N(0,1) bf16 queries, keys and values, and
    for each prompt ceil(len / PAGE) distinct pages of a randomly permuted pool."""
    lens = np.asarray(prompt_lens, dtype=np.int64)
    cu = np.zeros(lens.size + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    T = int(cu[-1])
    npg = (lens + PAGE - 1) // PAGE
    needed = int(npg.sum())
    num_pages = max(needed + 1, int(math.ceil(slack * needed)))
    phys = _rng(seed, cfg_id, 0, 5).permutation(num_pages)[:needed].astype(np.int32)
    off = np.zeros(lens.size + 1, dtype=np.int32)
    off[1:] = np.cumsum(npg)
    tid = 500 + cfg_id * 8
    return PrefillBatch(name=name, Hq=Hq, Hkv=Hkv, D=D, cu_seqlens=cu,
                        q=normal_bf16(T * Hq * D, seed, tid).reshape(T, Hq, D),
                        k=normal_bf16(T * Hkv * D, seed, tid + 1).reshape(T, Hkv, D),
                        v=normal_bf16(T * Hkv * D, seed, tid + 2).reshape(T, Hkv, D),
                        softmax_scale=np.float32(1.0 / math.sqrt(D)), num_pages=num_pages, page_offsets=off, pages=phys)


def make_prefill(config, seed=0, groups=None):
    """The prompts of a named configuration: one prompt per group, all of the configuration's prompt length."""
    cfg = CONFIGS[config]
    n = cfg["groups"] if groups is None else groups
    return build_prefill(config, cfg["Hq"], cfg["Hkv"], cfg["D"], [cfg["prompt"]] * n, seed=seed, cfg_id=cfg["id"])
