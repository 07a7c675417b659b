"""Prompt prefill on the GPU through the C ABI against the fp64 oracle: causal attention of packed prompts
(element by element at reduced sizes, whole prompts and sampled heads at the benchmark's sizes), the cache
write (bit-exact), and the hand-over to the decode step."""
import numpy as np
import pytest
import torch

import oracle
import paper_2507_01663_amd as ra
import workload
from gpu_util import ABS_TOL, LSE_TOL, REL_TOL, bits_to_bf16
from gpu_util import compare as compare_decode
from workload.gen import PAGE, bf16_bits_to_f32

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
OUT_ULP = 2.0 ** -8      # one bf16 unit in the last place, relative: the allowance for outputs that are not small


def compare(out, lse, ref_out, ref_lse, what=""):
    """The decode tolerances, with the element-wise bound widened by one bf16 ulp of the reference's magnitude."""
    return compare_decode(out, lse, ref_out, ref_lse, what, abs_rel=OUT_ULP)


@pytest.fixture(scope="module", params=["by prompt length", "one workgroup per block", "two workgroups per die that stay",
                                        "one per compute unit that stays"])
def dec(request):
    """Every test runs in the launch shape the library picks and in each of those it can be told to use: the results must
    not depend on how the blocks of query rows are dealt to workgroups (the setting is read when the context is made)."""
    import os
    value = {"by prompt length": None, "one workgroup per block": "0", "two workgroups per die that stay": "2",
             "one per compute unit that stays": "64"}[request.param]
    old = os.environ.get("ROLLOUT_ATTN_PREFILL_WGS_PER_DIE")
    if value is None:
        os.environ.pop("ROLLOUT_ATTN_PREFILL_WGS_PER_DIE", None)
    else:
        os.environ["ROLLOUT_ATTN_PREFILL_WGS_PER_DIE"] = value
    try:
        d = ra.Decoder(0)
    finally:
        if old is None:
            os.environ.pop("ROLLOUT_ATTN_PREFILL_WGS_PER_DIE", None)
        else:
            os.environ["ROLLOUT_ATTN_PREFILL_WGS_PER_DIE"] = old
    yield d
    d.close()


class DevicePrefill:
    def __init__(self, b, kv_dtype=None, max_len=None, poison=True):
        self.b = b
        self.q, self.k, self.v = bits_to_bf16(b.q, DEV), bits_to_bf16(b.k, DEV), bits_to_bf16(b.v, DEV)
        self.cu = torch.from_numpy(b.cu_seqlens).to(DEV)
        T = b.q.shape[0]
        self.out = torch.full((T, b.Hq, b.D), float("nan"), dtype=torch.bfloat16, device=DEV)
        self.lse = torch.full((T, b.Hq), float("nan"), dtype=torch.float32, device=DEV)
        pools = {}
        if kv_dtype is not None:
            shape = (b.num_pages, b.Hkv, PAGE, b.D)
            if kv_dtype == "bf16":
                self.k_pool = torch.full(shape, float("nan"), dtype=torch.bfloat16, device=DEV)
                self.v_pool = torch.full(shape, float("nan"), dtype=torch.bfloat16, device=DEV)
                self.k_scale = self.v_scale = None
            else:
                self.k_pool = torch.full(shape, 0x7F, dtype=torch.uint8, device=DEV)
                self.v_pool = torch.full(shape, 0x7F, dtype=torch.uint8, device=DEV)
                self.k_scale = torch.full((b.num_pages, b.Hkv), float("nan"), dtype=torch.float32, device=DEV)
                self.v_scale = torch.full((b.num_pages, b.Hkv), float("nan"), dtype=torch.float32, device=DEV)
            self.page_off = torch.from_numpy(b.page_offsets).to(DEV)
            self.pages = torch.from_numpy(b.pages).to(DEV) if b.pages.size else torch.zeros(1, dtype=torch.int32, device=DEV)
            pools = dict(k_pool=self.k_pool, v_pool=self.v_pool, k_scale=self.k_scale, v_scale=self.v_scale,
                         page_offsets=self.page_off, pages=self.pages)
        lens = b.lens
        self.c = ra.prefill_from_tensors(self.q, self.k, self.v, self.cu, int(lens.max()) if max_len is None and lens.size else (max_len or 0),
                                         self.out, self.lse, float(b.softmax_scale), **pools)

    def results(self):
        torch.cuda.synchronize()
        return self.out.float().cpu().numpy().astype(np.float64), self.lse.cpu().numpy().astype(np.float64)


def check_all(dec, b, what):
    d = DevicePrefill(b)
    dec.prefill(d.c)
    out, lse = d.results()
    ref_out, ref_lse = oracle.prefill(b.q, b.k, b.v, b.cu_seqlens, b.softmax_scale)
    return compare(out, lse, ref_out, ref_lse, what)


@pytest.mark.parametrize("Hq,Hkv,D,lens", [
    (28, 4, 128, [1, 15, 16, 17, 33, 255, 256, 257, 300, 0, 700]),     # around every tile, stage and block edge
    (8, 2, 64, [5, 64, 513, 31, 32]),
    (4, 4, 128, [129, 2, 511]),                                          # one query head per kv head
    (32, 2, 64, [100, 260]),                                             # sixteen
    (40, 8, 128, [48, 1024]),
])
def test_every_element_against_the_oracle(dec, Hq, Hkv, D, lens):
    b = workload.build_prefill("pf", Hq, Hkv, D, lens, seed=3)
    errs = check_all(dec, b, "prefill Hq=%d Hkv=%d D=%d lens=%s" % (Hq, Hkv, D, lens))
    print("errors (abs, row-rel, lse):", errs)


def test_large_scores_and_an_outlier_key(dec):
    # scores far from zero exercise the running maximum: a key early in the prompt that dominates, then is overtaken
    b = workload.build_prefill("pf", 8, 2, 128, [400], seed=5)
    k = bf16_bits_to_f32(b.k).copy()
    k[7] *= 6.0
    k[300] *= 9.0
    b.k = workload.f32_to_bf16_bits(k)
    check_all(dec, b, "outlier keys")


@pytest.mark.parametrize("D", [64, 128])
def test_keys_a_thousand_times_larger_than_the_rest(dec, D):
    # A key whose scores dwarf all others makes any disagreement between the reference point of the exponent and the
    # scores it is applied to overflow at once (the reference point comes from a maximum over fresh MFMA results; the
    # weights from the same results a little later).  One such key in the first stage, one at a stage edge, one in the
    # middle of a later block.
    b = workload.build_prefill("pf", 8, 2, D, [100, 700], seed=11)
    k = bf16_bits_to_f32(b.k).copy()
    for t in (6, 100 + 31, 100 + 32, 100 + 300, 100 + 511):
        k[t] *= 1000.0
    b.k = workload.f32_to_bf16_bits(k)
    check_all(dec, b, "dominant keys, D=%d" % D)


def test_no_prompts_and_empty_prompts(dec):
    b = workload.build_prefill("pf", 8, 2, 64, [0, 0], seed=1)
    d = DevicePrefill(b, max_len=0)
    dec.prefill(d.c)            # nothing to do, nothing touched
    torch.cuda.synchronize()
    b = workload.build_prefill("pf", 8, 2, 64, [0, 40, 0], seed=1)
    check_all(dec, b, "empty prompts around one")


def test_bound_on_the_prompt_length_sizes_the_launch(dec):
    # a bound above the real lengths costs nothing but idle workgroups; one below them leaves the tail of a prompt
    # untouched (whole blocks of 256 query rows), and what is computed is still right
    b = workload.build_prefill("pf", 8, 2, 128, [300, 40], seed=2)
    ref_out, ref_lse = oracle.prefill(b.q, b.k, b.v, b.cu_seqlens, b.softmax_scale)
    d = DevicePrefill(b, max_len=2000)
    dec.prefill(d.c)
    compare(*d.results(), ref_out, ref_lse, "generous bound")
    d = DevicePrefill(b, max_len=200)
    dec.prefill(d.c)
    out, lse = d.results()
    compare(out[:256], lse[:256], ref_out[:256], ref_lse[:256], "first block of the long prompt")
    compare(out[300:], lse[300:], ref_out[300:], ref_lse[300:], "the short prompt")
    assert np.isnan(out[256:300]).all() and np.isnan(lse[256:300]).all()


def test_benchmark_size_whole_prompts(dec):
    # the launch bench.py times (32 prompts of 512, 7B head shape); three prompts in full against the oracle
    b = workload.make_prefill("grpo7b", seed=0)
    d = DevicePrefill(b)
    dec.prefill(d.c)
    out, lse = d.results()
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    for g in (0, 13, 31):
        a, e = int(b.cu_seqlens[g]), int(b.cu_seqlens[g + 1])
        cu = np.array([0, e - a], dtype=np.int32)
        ref_out, ref_lse = oracle.prefill(b.q[a:e], b.k[a:e], b.v[a:e], cu, b.softmax_scale)
        compare(out[a:e], lse[a:e], ref_out, ref_lse, "grpo7b prompt %d" % g)


@pytest.mark.parametrize("config,groups", [("tail32b", 64), ("stream72b", 16)])
def test_benchmark_size_sampled_heads(dec, config, groups):
    # full launch; the oracle takes two prompts with two query heads each (and the kv heads they use)
    b = workload.make_prefill(config, seed=0, groups=groups)
    d = DevicePrefill(b)
    dec.prefill(d.c)
    out, lse = d.results()
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    G = b.Hq // b.Hkv
    for g, heads in ((1, (0, b.Hq - 1)), (groups - 1, (G, 2 * G + 1))):
        a, e = int(b.cu_seqlens[g]), int(b.cu_seqlens[g + 1])
        cu = np.array([0, e - a], dtype=np.int32)
        for h in heads:
            kv = h // G
            ref_out, ref_lse = oracle.prefill(b.q[a:e, h:h + 1], b.k[a:e, kv:kv + 1], b.v[a:e, kv:kv + 1], cu, b.softmax_scale)
            compare(out[a:e, h:h + 1], lse[a:e, h:h + 1], ref_out, ref_lse, "%s prompt %d head %d" % (config, g, h))


def expected_pools(b, kv_dtype):
    """What the cache write must leave in pools that started out as poison: the oracle's cache write
    (oracle.prefill_write, pinned on the CPU in tests/test_prefill_oracle_pins.py)."""
    shape = (b.num_pages, b.Hkv, PAGE, b.D)
    if kv_dtype == "bf16":
        kp, vp = np.full(shape, 0x7FC0, dtype=np.uint16), np.full(shape, 0x7FC0, dtype=np.uint16)
        ks = vs = None
    else:
        kp, vp = np.full(shape, 0x7F, dtype=np.uint8), np.full(shape, 0x7F, dtype=np.uint8)
        ks, vs = np.full(shape[:2], np.nan, dtype=np.float32), np.full(shape[:2], np.nan, dtype=np.float32)
    oracle.prefill_write(b.k, b.v, b.cu_seqlens, b.page_offsets, b.pages, kp, vp, ks, vs)
    return kp, vp, ks, vs


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8_e4m3"])
@pytest.mark.parametrize("D", [64, 128])
def test_cache_write_is_bit_exact(dec, kv_dtype, D):
    b = workload.build_prefill("pf", 8, 2, D, [1, 16, 17, 100, 0, 260], seed=7)
    k = bf16_bits_to_f32(b.k).copy()
    k[20:36] = 0.0                    # a page of zeros: scale 1
    k[40] *= 1000.0                   # and one with a large row
    b.k = workload.f32_to_bf16_bits(k)
    d = DevicePrefill(b, kv_dtype=kv_dtype)
    dec.prefill(d.c)
    torch.cuda.synchronize()
    kp, vp, ks, vs = expected_pools(b, kv_dtype)
    view = (lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)) if kv_dtype == "bf16" else (lambda t: t.cpu().numpy())
    np.testing.assert_array_equal(view(d.k_pool), kp)
    np.testing.assert_array_equal(view(d.v_pool), vp)
    if kv_dtype != "bf16":
        np.testing.assert_array_equal(d.k_scale.cpu().numpy().view(np.uint32), ks.view(np.uint32))
        np.testing.assert_array_equal(d.v_scale.cpu().numpy().view(np.uint32), vs.view(np.uint32))
    # and the attention was computed as well
    out, lse = d.results()
    ref_out, ref_lse = oracle.prefill(b.q, b.k, b.v, b.cu_seqlens, b.softmax_scale)
    compare(out, lse, ref_out, ref_lse, "prefill with cache write")


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8_e4m3"])
def test_cache_write_into_pools_that_are_views(dec, kv_dtype):
    # K and V interleaved per page in one allocation, with room between the token rows: the write goes through the strides
    b = workload.build_prefill("pf", 8, 2, 128, [70, 33], seed=13)
    d = DevicePrefill(b, kv_dtype=kv_dtype)
    pad = 32 if kv_dtype == "bf16" else 64
    both = torch.zeros((b.num_pages, 2, b.Hkv, PAGE, b.D + pad), dtype=d.k_pool.dtype, device=DEV)
    both[..., :b.D] = torch.stack([d.k_pool, d.v_pool], dim=1)
    kp, vp = both[:, 0, :, :, :b.D], both[:, 1, :, :, :b.D]
    d.c = ra.prefill_from_tensors(d.q, d.k, d.v, d.cu, int(b.lens.max()), d.out, d.lse, float(b.softmax_scale), k_pool=kp, v_pool=vp,
                                  k_scale=d.k_scale, v_scale=d.v_scale, page_offsets=d.page_off, pages=d.pages)
    assert d.c.kv_stride_token == b.D + pad and d.c.kv_stride_page == 2 * b.Hkv * PAGE * (b.D + pad)
    dec.prefill(d.c)
    torch.cuda.synchronize()
    ek, ev, eks, evs = expected_pools(b, kv_dtype)
    view = (lambda t: t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)) if kv_dtype == "bf16" else (lambda t: t.contiguous().cpu().numpy())
    np.testing.assert_array_equal(view(kp), ek)
    np.testing.assert_array_equal(view(vp), ev)
    assert (both[..., b.D:] == 0).all()          # nothing landed between the rows
    if kv_dtype != "bf16":
        np.testing.assert_array_equal(d.k_scale.cpu().numpy().view(np.uint32), eks.view(np.uint32))
        np.testing.assert_array_equal(d.v_scale.cpu().numpy().view(np.uint32), evs.view(np.uint32))


def test_cache_write_skips_missing_and_invalid_pages(dec):
    b = workload.build_prefill("pf", 4, 2, 64, [50, 50], seed=9)
    # prompt 0 keeps only two of its four pages; prompt 1 has one page id out of range
    keep = np.concatenate([b.pages[0:2], b.pages[4:8]]).astype(np.int32)
    keep[3] = b.num_pages + 5
    b.pages = keep
    b.page_offsets = np.array([0, 2, 6], dtype=np.int32)
    d = DevicePrefill(b, kv_dtype="bf16")
    dec.prefill(d.c)
    torch.cuda.synchronize()
    kp, vp, _, _ = expected_pools(b, "bf16")
    np.testing.assert_array_equal(d.k_pool.view(torch.int16).cpu().numpy().view(np.uint16), kp)
    np.testing.assert_array_equal(d.v_pool.view(torch.int16).cpu().numpy().view(np.uint16), vp)


def test_decode_of_the_last_prompt_token_over_the_written_pages(dec):
    # prefill writes the prompts' pages; a decode step whose query is each prompt's last token over exactly those
    # pages must give that token's prefill output (both are checked against their own oracles elsewhere; here
    # the two kernels meet through the cache)
    b = workload.build_prefill("pf", 28, 4, 128, [512, 100, 333], seed=4)
    d = DevicePrefill(b, kv_dtype="bf16")
    dec.prefill(d.c)
    out, lse = d.results()
    lens = b.lens
    last = (b.cu_seqlens[1:] - 1).astype(np.int64)
    n = lens.size
    width = int(((lens + PAGE - 1) // PAGE).max())
    bt = np.full((n, width), -1, dtype=np.int32)
    for g in range(n):
        ids = b.pages[b.page_offsets[g]:b.page_offsets[g + 1]]
        bt[g, :ids.size] = ids
    q = d.q[torch.from_numpy(last).to(DEV)].contiguous()
    o2 = torch.full((n, b.Hq, b.D), float("nan"), dtype=torch.bfloat16, device=DEV)
    l2 = torch.full((n, b.Hq), float("nan"), dtype=torch.float32, device=DEV)
    prob = ra.problem_from_tensors(q, d.k_pool, d.v_pool, torch.from_numpy(bt).to(DEV), torch.from_numpy(lens.astype(np.int32)).to(DEV),
                                   o2, l2, float(b.softmax_scale))
    dec.decode(prob)
    torch.cuda.synchronize()
    dout = o2.float().cpu().numpy().astype(np.float64)
    dlse = l2.cpu().numpy().astype(np.float64)
    assert np.abs(dout - out[last]).max() <= 2 * ABS_TOL
    assert np.abs(dlse - lse[last]).max() <= 2 * LSE_TOL
    num = np.sqrt(((dout - out[last]) ** 2).sum(-1))
    den = np.sqrt((out[last] ** 2).sum(-1))
    assert (num / den).max() <= 2 * REL_TOL


def test_rejected_arguments(dec):
    b = workload.build_prefill("pf", 8, 2, 64, [40], seed=1)
    d = DevicePrefill(b)
    for field, value, status in (("Hq", 7, ra.RA_ERR_INVALID_ARG), ("D", 96, ra.RA_ERR_UNSUPPORTED), ("q", None, ra.RA_ERR_INVALID_ARG),
                                 ("softmax_scale", float("nan"), ra.RA_ERR_INVALID_ARG), ("num_prompts", -1, ra.RA_ERR_INVALID_ARG)):
        old = getattr(d.c, field)
        setattr(d.c, field, value)
        with pytest.raises(ra.RolloutAttnError) as e:
            dec.prefill(d.c)
        assert e.value.status == status, field
        setattr(d.c, field, old)
    dec.prefill(d.c)
    torch.cuda.synchronize()
