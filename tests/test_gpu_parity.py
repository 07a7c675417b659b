"""GPU parity: the HIP library, called through its C ABI, against the fp64 oracle on the same seeded inputs.
Integer work (page arithmetic, gather order) must be bit-exact; outputs within max-abs 1e-2 and per-row
relative 1e-2, log-sum-exp within 1e-3 (bf16 inputs)."""
import ctypes
import sys

import numpy as np
import pytest
import torch

import oracle
import workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dec():
    import paper_2507_01663_amd as ra
    d = ra.Decoder(0)
    yield d
    d.close()


def run(dec, p, flags=0, use_hint=True):
    from gpu_util import DeviceProblem
    dp = DeviceProblem(p, flags=flags, use_hint=use_hint)
    dec.decode(dp.c)
    return dp


def log(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("name", ["tiny", "midd64", "mid7b", "mid32b", "mid72b"])
def test_parity_element_by_element(dec, name):
    from gpu_util import compare
    p = workload.make_problem(name, seed=0)
    log("case", name, "B", p.B, "lens", int(p.seq_lens.min()), int(p.seq_lens.max()))
    ref_out, ref_lse = oracle.decode(p)
    dp = run(dec, p)
    errs = compare(*dp.results(), ref_out, ref_lse, name)
    log(name, "abs %.2e rel %.2e lse %.2e" % errs)


@pytest.mark.parametrize("name", ["tiny", "midd64", "mid7b", "mid32b", "mid72b"])
def test_fp8_kv_parity_element_by_element(dec, name):
    """K/V stored as e4m3 codes with per-page-per-head fp32 scales; the oracle dequantises in fp64."""
    from gpu_util import compare
    p = workload.make_problem(name, seed=0, kv_dtype="fp8_e4m3")
    log("case", p.name, "B", p.B, "lens", int(p.seq_lens.min()), int(p.seq_lens.max()))
    ref_out, ref_lse = oracle.decode(p)
    errs = compare(*run(dec, p).results(), ref_out, ref_lse, p.name)
    log(p.name, "abs %.2e rel %.2e lse %.2e" % errs)
    errs = compare(*run(dec, p, use_hint=False).results(), ref_out, ref_lse, p.name + " no hint")


def test_fp8_every_code_decodes_exactly(dec):
    """One key per sequence (softmax weight 1), V rows holding every finite e4m3 code, scale 1: the output must be
    the code's value rounded to bf16, i.e. exactly the value."""
    from gpu_util import compare
    p = workload.build_problem("codes", 4, 4, 64, [0], 16, [1] * 16, kv_dtype="fp8_e4m3", seed=7, poison=False)
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)     # 254 finite codes
    vals = np.resize(codes, 16 * 4 * 64).reshape(16, 4, 64)
    for b in range(16):
        pg = p.block_table[b, 0]
        p.v_pool[pg, :, 0, :] = vals[b]
        p.k_pool[pg, :, 0, :] = vals[(b + 5) % 16]
    p.k_scale[:] = 2.0 ** -9
    p.v_scale[:] = 1.0
    ref_out, ref_lse = oracle.decode(p)
    out, lse = run(dec, p).results()
    tab = oracle.e4m3_decode_table()
    assert np.array_equal(ref_out, np.repeat(tab[vals][:, :, None, :], 1, axis=2).reshape(16, 4, 64))
    assert np.array_equal(out, ref_out)                 # exact: every e4m3 value is a bf16 value
    compare(out, lse, ref_out, ref_lse, "codes")


@pytest.mark.parametrize("name", ["tiny", "mid7b"])
def test_hint_off_and_flag_give_the_same_answer(dec, name):
    import paper_2507_01663_amd as ra
    from gpu_util import compare
    p = workload.make_problem(name, seed=1)
    ref_out, ref_lse = oracle.decode(p)
    for kw in (dict(use_hint=False), dict(flags=ra.RA_FLAG_NO_PREFIX_SHARING), dict(flags=ra.RA_FLAG_VALIDATE)):
        dp = run(dec, p, **kw)
        compare(*dp.results(), ref_out, ref_lse, "%s %s" % (name, kw))


def test_streaming_steps_rebuild_the_table(dec):
    from gpu_util import compare
    p0 = workload.make_problem("mid72b", seed=0, step=0)
    pool = (p0.k_pool, p0.v_pool, None, None)
    for step in (1, 5, 7):
        p = workload.make_problem("mid72b", seed=0, step=step, pool=pool, num_pages=p0.num_pages)
        ref_out, ref_lse = oracle.decode(p)
        dp = run(dec, p)
        compare(*dp.results(), ref_out, ref_lse, "mid72b step %d" % step)


def test_edge_lengths(dec):
    from gpu_util import compare
    # empty sequences, single token, exact page multiples, one past a page, a group whose members are all empty
    lens = [0, 1, 15, 16, 17, 31, 32, 33, 0, 0, 64, 65, 127, 128, 129, 300]
    p = workload.build_problem("edge", 8, 2, 128, [0, 0], 8, lens, seed=2)
    ref_out, ref_lse = oracle.decode(p)
    dp = run(dec, p)
    out, lse = dp.results()
    compare(out, lse, ref_out, ref_lse, "edge")
    assert (out[0] == 0).all() and np.isneginf(lse[0]).all()
    # prompt not page aligned (20 tokens -> 1 shared page), a member shorter than... every member holds the prefix
    p = workload.build_problem("edge2", 6, 2, 64, [20, 16, 48], 3, [0, 5, 40, 1, 0, 29, 0, 0, 0], seed=3)
    ref_out, ref_lse = oracle.decode(p)
    compare(*run(dec, p).results(), ref_out, ref_lse, "edge2")


def test_member_shorter_than_prefix_falls_back(dec):
    from gpu_util import DeviceProblem, compare
    p = workload.build_problem("short", 4, 2, 64, [64], 4, [0, 10, 0, 33], seed=4)
    # cut sequence 2 down to 40 tokens: it no longer holds the whole 4-page prefix
    p.seq_lens[2] = 40
    ref_out, ref_lse = oracle.decode(p)
    compare(*run(dec, p).results(), ref_out, ref_lse, "short member")


def test_scattered_group_ids_and_ungrouped(dec):
    from gpu_util import compare
    p = workload.build_problem("scatter", 8, 4, 128, [32, 32, 32], 4, list(range(5, 17)), seed=5)
    # relabel: group ids need not be contiguous in b; one sequence opts out with -1
    perm = np.random.default_rng(0).permutation(p.B)
    for name in ("q", "block_table", "seq_lens", "seq_group"):
        setattr(p, name, np.ascontiguousarray(getattr(p, name)[perm]))
    p.seq_group[3] = -1
    ref_out, ref_lse = oracle.decode(p)
    compare(*run(dec, p).results(), ref_out, ref_lse, "scattered")


def test_many_members_need_several_prefix_rows(dec):
    from gpu_util import compare
    # 16 members x 8 heads per kv head = 128 query rows on the shared pages: more than one work row carries
    p = workload.build_problem("wide", 16, 2, 128, [96], 16, list(range(0, 160, 10)), seed=6)
    ref_out, ref_lse = oracle.decode(p)
    compare(*run(dec, p).results(), ref_out, ref_lse, "wide group")


def test_batch_beyond_the_schedules_lds_tables(dec):
    from gpu_util import compare
    # more sequences (and groups) than the schedule kernels keep in LDS: their tables then live in the workspace
    ngroups, R = 1100, 2
    rng = np.random.default_rng(9)
    resp = rng.integers(0, 40, size=ngroups * R)
    p = workload.build_problem("large_b", 4, 2, 64, [16] * ngroups, R, resp, seed=9)
    assert p.B > 2048 and ngroups <= 2048
    ref_out, ref_lse = oracle.decode(p)
    compare(*run(dec, p).results(), ref_out, ref_lse, "B = %d" % p.B)
    compare(*run(dec, p, use_hint=False).results(), ref_out, ref_lse, "B = %d, no hint" % p.B)
    # and more groups than fit as well
    ngroups = 2100
    resp = rng.integers(0, 40, size=ngroups)
    p = workload.build_problem("large_g", 4, 2, 64, [16] * ngroups, 1, resp, seed=10)
    ref_out, ref_lse = oracle.decode(p)
    compare(*run(dec, p).results(), ref_out, ref_lse, "groups = %d" % ngroups)


@pytest.fixture(scope="module")
def dec_sched():
    """A context that always launches the schedule kernels (the path of batches too large for the attention waves to
    plan for themselves); the setting is read when the context is made."""
    import os
    import paper_2507_01663_amd as ra
    old = os.environ.get("ROLLOUT_ATTN_SELF_PLAN")
    os.environ["ROLLOUT_ATTN_SELF_PLAN"] = "0"
    try:
        d = ra.Decoder(0)
    finally:
        if old is None:
            os.environ.pop("ROLLOUT_ATTN_SELF_PLAN", None)
        else:
            os.environ["ROLLOUT_ATTN_SELF_PLAN"] = old
    yield d
    d.close()


@pytest.mark.parametrize("name,kv", [("tiny", "bf16"), ("mid7b", "bf16"), ("mid32b", "fp8_e4m3"), ("mid72b", "bf16"), ("grpo7b", "bf16")])
def test_parity_with_the_schedule_kernels(dec_sched, dec, name, kv):
    """Small batches normally take the path where every attention wave plans its own span; the same batches through
    the schedule kernels must give the same answer within tolerance (the spans are the same, so in fact the same bytes)."""
    from gpu_util import compare
    p = workload.make_problem(name, seed=0, kv_dtype=kv)
    ref = oracle.decode(p)
    a = run(dec_sched, p)
    compare(*a.results(), *ref, "%s %s (schedule kernels)" % (name, kv))
    b = run(dec, p)
    torch.cuda.synchronize()
    assert torch.equal(a.out.view(torch.int16), b.out.view(torch.int16)) and torch.equal(a.lse, b.lse)


def test_phase_timing_reports_only_the_launches_made(dec_sched, dec):
    """The per-phase event timing: a batch planned inside the attention kernel has no schedule phase (0), the same
    batch through the schedule kernels has one; attention and merge always do.  Results are not touched by it."""
    import paper_2507_01663_amd as ra
    p = workload.make_problem("mid7b", seed=0)
    plain = run(dec, p)
    torch.cuda.synchronize()
    for d, has_schedule in ((dec, False), (dec_sched, True)):
        with pytest.raises(ra.RolloutAttnError):
            ra.rollout_attn_get_timing(d.ctx)             # nothing timed yet
        ra.rollout_attn_set_timing(d.ctx, True)
        try:
            timed = run(d, p)
            ms = ra.rollout_attn_get_timing(d.ctx)
        finally:
            ra.rollout_attn_set_timing(d.ctx, False)
        assert len(ms) == 3 and ms[1] > 0 and ms[2] > 0 and all(x < 100 for x in ms), ms
        assert (ms[0] > 0) == has_schedule, ms
        assert torch.equal(timed.out.view(torch.int16), plain.out.view(torch.int16)) and torch.equal(timed.lse, plain.lse)


@pytest.fixture(scope="module")
def dec_few_waves():
    """A context with one attention workgroup per compute unit instead of four: four times longer spans."""
    import os
    import paper_2507_01663_amd as ra
    old = os.environ.get("ROLLOUT_ATTN_WAVES_PER_CU")
    os.environ["ROLLOUT_ATTN_WAVES_PER_CU"] = "1"
    try:
        d = ra.Decoder(0)
    finally:
        if old is None:
            os.environ.pop("ROLLOUT_ATTN_WAVES_PER_CU", None)
        else:
            os.environ["ROLLOUT_ATTN_WAVES_PER_CU"] = old
    yield d
    d.close()


def test_spans_with_more_segments_than_a_wave_lists_at_once(dec_few_waves):
    """A few very long sequences make the spans long, and hundreds of very short ones then fall into single spans
    (about 150 segments each here): a wave that plans for itself lists at most 64 (head dim 64) or 128 segments at a
    time and has to plan again from where it stopped; shared-prefix rows of many members (one query head per kv head)
    take several records each."""
    from gpu_util import compare
    dec = dec_few_waves
    for D, Hkv, Hq in ((64, 8, 8), (128, 4, 4)):
        rng = np.random.default_rng(31 + D)
        ngroups, R = 6, 70
        resp = rng.integers(1, 3, size=ngroups * R)          # one or two tokens beyond the prompt
        resp[::R] = 111000                                    # one long member per group
        p = workload.build_problem("fragments", Hq, Hkv, D, [16] * ngroups, R, resp, seed=31)
        assert p.B == 420
        log("fragments D", D, "pages", p.num_pages)
        ref_out, ref_lse = oracle.decode(p)
        compare(*run(dec, p).results(), ref_out, ref_lse, "fragments D = %d" % D)
        compare(*run(dec, p, use_hint=False).results(), ref_out, ref_lse, "fragments D = %d, no hint" % D)


def test_sixteen_query_heads_per_kv_head(dec):
    from gpu_util import compare
    for D in (64, 128):
        p = workload.build_problem("g16", 32, 2, D, [48, 16], 3, [0, 5, 77, 130, 16, 33], seed=12)
        ref_out, ref_lse = oracle.decode(p)
        compare(*run(dec, p).results(), ref_out, ref_lse, "G = 16, D = %d" % D)


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8_e4m3"])
def test_gather_is_bit_exact(dec, kv_dtype):
    """rollout_attn_debug_gather against oracle.gather, raw stored elements (bf16 bit patterns or e4m3 codes)."""
    from gpu_util import DeviceProblem
    fp8 = kv_dtype != "bf16"
    for name in ("tiny", "mid32b"):
        p = workload.make_problem(name, seed=0, kv_dtype=kv_dtype)
        dp = DeviceProblem(p)
        rng = np.random.default_rng(0)
        pairs = [(b, kv) for b in range(p.B) for kv in range(p.Hkv)]
        if len(pairs) > 24:
            pairs = [pairs[i] for i in rng.choice(len(pairs), 24, replace=False)]
        for b, kv in pairs:
            L = int(p.seq_lens[b])
            k_out = torch.zeros((L, p.D), dtype=torch.uint8 if fp8 else torch.bfloat16, device="cuda:0")
            v_out = torch.zeros_like(k_out)
            dec.debug_gather(dp.c, b, kv, k_out, v_out)
            torch.cuda.synchronize()
            rk, rv, _ = oracle.gather(p, b, kv)
            host = (lambda t: t.cpu().numpy()) if fp8 else (lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16))
            assert rk.dtype == (np.uint8 if fp8 else np.uint16)
            assert np.array_equal(host(k_out), rk), (name, kv_dtype, b, kv)
            assert np.array_equal(host(v_out), rv), (name, kv_dtype, b, kv)


def test_page_arithmetic_through_the_attention_kernels(dec):
    """Values that encode (page, slot): a wrong page or slot in the attention path changes the result grossly."""
    from gpu_util import compare
    p = workload.make_problem("mid7b", seed=2)
    pg = np.arange(p.num_pages, dtype=np.float32)[:, None, None, None]
    sl = np.arange(16, dtype=np.float32)[None, None, :, None]
    hd = np.arange(p.Hkv, dtype=np.float32)[None, :, None, None]
    d = np.arange(p.D, dtype=np.float32)[None, None, None, :]
    nan_k, nan_v = p.k_pool == workload.BF16_NAN, p.v_pool == workload.BF16_NAN
    p.k_pool[:] = workload.f32_to_bf16_bits(np.sin(0.37 * pg + 1.3 * sl + hd + 0.05 * d))
    p.v_pool[:] = workload.f32_to_bf16_bits((1.0 + 0.5 * np.cos(0.11 * pg + 0.7 * sl + 2 * hd)) * (0.5 + d / 256))
    p.k_pool[nan_k] = workload.BF16_NAN
    p.v_pool[nan_v] = workload.BF16_NAN
    ref_out, ref_lse = oracle.decode(p)
    compare(*run(dec, p).results(), ref_out, ref_lse, "encoded pool")


def test_two_runs_are_byte_identical(dec):
    p = workload.make_problem("mid32b", seed=3)
    a = run(dec, p)
    o1, l1 = a.out.clone(), a.lse.clone()
    b = run(dec, p)
    torch.cuda.synchronize()
    assert torch.equal(o1.view(torch.int16), b.out.view(torch.int16)) and torch.equal(l1, b.lse)


def test_interleaved_group_members_are_byte_identical_run_to_run(dec):
    """Members of a group scattered over the batch (every fourth sequence, across the waves and blocks of the
    schedule kernel) and many more of them than one shared-prefix row carries: which row a member joins must be a
    function of the inputs, so repeated runs agree bit for bit (and with the oracle within tolerance)."""
    from gpu_util import compare
    ngroups, R = 4, 70
    rng = np.random.default_rng(21)
    p = workload.build_problem("interleaved", 14, 2, 128, [64] * ngroups, R, rng.integers(0, 200, size=ngroups * R), seed=21)
    order = np.array([g * R + r for r in range(R) for g in range(ngroups)])          # b' = r * ngroups + g
    for name in ("q", "block_table", "seq_lens", "seq_group"):
        setattr(p, name, np.ascontiguousarray(getattr(p, name)[order]))
    assert p.B == 280 and (p.seq_group[:8] == [0, 1, 2, 3, 0, 1, 2, 3]).all()
    ref_out, ref_lse = oracle.decode(p)
    first = None
    for rep in range(6):
        dp = run(dec, p)
        torch.cuda.synchronize()
        got = (dp.out.view(torch.int16).clone(), dp.lse.clone())
        if first is None:
            first = got
            compare(*dp.results(), ref_out, ref_lse, "interleaved members")
        else:
            assert torch.equal(first[0], got[0]) and torch.equal(first[1], got[1]), "run %d differs from run 0" % rep


def test_strided_pool_layout(dec):
    """Pools that are views of a larger allocation (K and V interleaved per page) use the stride arguments."""
    from gpu_util import DeviceProblem, bits_to_bf16, compare
    import paper_2507_01663_amd as ra
    p = workload.make_problem("midd64", seed=4)
    ref_out, ref_lse = oracle.decode(p)
    dp = DeviceProblem(p)
    both = torch.stack([dp.k_pool, dp.v_pool], dim=1).contiguous()      # [pages, 2, Hkv, 16, D]
    dp.k_pool, dp.v_pool = both[:, 0], both[:, 1]
    dp.set()
    assert dp.c.kv_stride_page == 2 * p.Hkv * 16 * p.D
    dec.decode(dp.c)
    compare(*dp.results(), ref_out, ref_lse, "strided")


def test_validate_flag_reports_bad_device_data(dec):
    import paper_2507_01663_amd as ra
    from gpu_util import DeviceProblem
    p = workload.make_problem("midd64", seed=5)
    dp = DeviceProblem(p, flags=ra.RA_FLAG_VALIDATE)
    dp.block_table[2, 1] = p.num_pages + 7
    with pytest.raises(ra.RolloutAttnError) as e:
        dec.decode(dp.c)
    assert e.value.status == ra.RA_ERR_OUT_OF_RANGE and "page id" in str(e.value)
    dp.block_table[2, 1] = int(p.block_table[2, 1])
    dp.seq_lens[0] = p.max_pages_per_seq * 16 + 1
    with pytest.raises(ra.RolloutAttnError) as e:
        dec.decode(dp.c)
    assert e.value.status == ra.RA_ERR_OUT_OF_RANGE and "length" in str(e.value)
    dp.seq_lens[0] = int(p.seq_lens[0])
    dp.block_table[1, 0] = int(p.block_table[5, 1])          # member row no longer starts with the shared page
    with pytest.raises(ra.RolloutAttnError) as e:
        dec.decode(dp.c)
    assert e.value.status == ra.RA_ERR_OUT_OF_RANGE


def test_workspace_too_small_and_bad_arguments(dec):
    import paper_2507_01663_amd as ra
    from gpu_util import DeviceProblem
    p = workload.make_problem("tiny")
    dp = DeviceProblem(p)
    ws = dec.workspace(dp.c)
    with pytest.raises(ra.RolloutAttnError) as e:
        ra.rollout_attn_decode(dec.ctx, dp.c, ctypes.c_void_p(ws.data_ptr()), 1024, None)
    assert e.value.status == ra.RA_ERR_WORKSPACE_TOO_SMALL
    dp.c.D = 96
    with pytest.raises(ra.RolloutAttnError) as e:
        dec.decode(dp.c)
    assert e.value.status == ra.RA_ERR_UNSUPPORTED
    # outputs untouched by rejected calls
    assert torch.isnan(dp.out.float()).all()


def test_full_size_grpo7b_against_oracle(dec):
    """The benchmark workload at full size, every row (the oracle needs about a second for it)."""
    from gpu_util import compare
    p = workload.make_problem("grpo7b", seed=0)
    log("grpo7b: kv tokens", p.kv_tokens(), "pages", p.num_pages)
    ref_out, ref_lse = oracle.decode(p)
    dp = run(dec, p)
    errs = compare(*dp.results(), ref_out, ref_lse, "grpo7b")
    log("grpo7b abs %.2e rel %.2e lse %.2e" % errs)
    dp2 = run(dec, p, use_hint=False)
    compare(*dp2.results(), ref_out, ref_lse, "grpo7b no hint")


def test_full_size_grpo7b_fp8_against_oracle(dec):
    from gpu_util import compare
    p = workload.make_problem("grpo7b", seed=0, kv_dtype="fp8_e4m3")
    ref_out, ref_lse = oracle.decode(p)
    errs = compare(*run(dec, p).results(), ref_out, ref_lse, "grpo7b fp8")
    log("grpo7b fp8 abs %.2e rel %.2e lse %.2e" % errs)


def test_full_size_tail32b_against_oracle(dec):
    """32B-shaped long-tail batch at full size (B=512, lognormal lengths up to 17408 tokens): every (b, h) row."""
    from gpu_util import compare
    p = workload.make_problem("tail32b", seed=0)
    log("tail32b: kv tokens", p.kv_tokens(), "pages", p.num_pages, "max len", int(p.seq_lens.max()))
    ref_out, ref_lse = oracle.decode(p)
    log("tail32b: oracle done")
    dp = run(dec, p)
    errs = compare(*dp.results(), ref_out, ref_lse, "tail32b")
    log("tail32b %d rows: abs %.2e rel %.2e lse %.2e" % ((p.B * p.Hq,) + errs))


def test_full_size_stream72b_steps(dec):
    """72B-shaped streaming batch at full size: static pool, lengths advance and the block table is re-drawn every
    step; every (b, h) row of steps 0, 1, 31 and 63 is checked."""
    from gpu_util import DeviceProblem, bits_to_bf16, compare
    p0 = workload.make_problem("stream72b", seed=0, step=0)
    log("stream72b: kv tokens", p0.kv_tokens(), "pages", p0.num_pages)
    cfg = workload.CONFIGS["stream72b"]
    width = (cfg["prompt"] + cfg["resp_max"] + cfg["steps"]) // 16 + 1       # room for every step of the run
    bt0 = np.full((p0.B, width), -1, dtype=np.int32)
    bt0[:, :p0.block_table.shape[1]] = p0.block_table
    p0.block_table, p0.max_pages_per_seq = bt0, width
    dp = DeviceProblem(p0)
    pool = (p0.k_pool, p0.v_pool, None, None)
    for step in (0, 1, 31, 63):
        p = p0 if step == 0 else workload.make_problem("stream72b", seed=0, step=step, pool=pool, num_pages=p0.num_pages,
                                                        make_values=False)
        if step:
            # same pool on the device; new q, lengths, table and prefix list
            p.q = workload.normal_bf16(p.B * p.Hq * p.D, 0, 99 + step).reshape(p.B, p.Hq, p.D)
            dp.p = p
            dp.q = bits_to_bf16(p.q, "cuda:0")
            assert p.block_table.shape[1] <= width
            bt = np.full((p.B, width), -1, dtype=np.int32)
            bt[:, :p.block_table.shape[1]] = p.block_table
            dp.block_table.copy_(torch.from_numpy(bt))
            dp.seq_lens.copy_(torch.from_numpy(p.seq_lens))
            dp.pfx_pages.copy_(torch.from_numpy(p.prefix_pages))
            dp.out.fill_(float("nan"))
            dp.set()
            p.block_table, p.max_pages_per_seq = bt, width
        dec.decode(dp.c)
        out, lse = dp.results()
        log("stream72b step %d: GPU done, oracle over all %d rows ..." % (step, p.B * p.Hq))
        ref_out, ref_lse = oracle.decode(p)
        errs = compare(out, lse, ref_out, ref_lse, "stream72b step %d" % step)
        log("stream72b step %d, %d rows: abs %.2e rel %.2e lse %.2e" % ((step, p.B * p.Hq) + errs))


def test_schedule_reused_for_another_layer(dec):
    import paper_2507_01663_amd as ra
    from gpu_util import DeviceProblem, compare
    # the layers of one decode step share lengths and groups, not queries, pools or page ids: the second problem has
    # its own of each and runs on the first one's schedule
    p1 = workload.make_problem("mid7b", seed=1)
    p2 = workload.make_problem("mid7b", seed=1)
    p2.q = workload.normal_bf16(p2.q.size, 77, 1).reshape(p2.q.shape)
    perm = np.random.default_rng(5).permutation(p2.num_pages).astype(np.int32)      # the same cache at other page ids
    inv = np.empty_like(perm)
    inv[perm] = np.arange(p2.num_pages, dtype=np.int32)
    p2.k_pool, p2.v_pool = p1.k_pool[inv].copy(), p1.v_pool[inv].copy()
    p2.block_table = np.where(p1.block_table >= 0, perm[np.maximum(p1.block_table, 0)], -1).astype(np.int32)
    p2.prefix_pages = perm[p1.prefix_pages]
    d1, d2 = DeviceProblem(p1), DeviceProblem(p2, flags=ra.RA_FLAG_REUSE_SCHEDULE)
    dec.decode(d1.c)
    dec.decode(d2.c)
    compare(*d1.results(), *oracle.decode(p1), "layer 1")
    compare(*d2.results(), *oracle.decode(p2), "layer 2 on layer 1's schedule")


@pytest.mark.parametrize("which", ["self-planned", "schedule kernels", "few waves"])
def test_random_batches_against_the_oracle(dec, dec_sched, dec_few_waves, which):
    """Seeded random shapes: head counts, head dim, group sizes, prompts that are not whole pages, empty and one-token
    responses beside long ones, relabelled and missing group ids, both pool types, hint on and off, and a second call on
    the first one's schedule.  Every element against the oracle, on each of the schedule's three paths.
    Sequences of one to three tokens do not average: their outputs are as large as single V entries (up to about 4.5
    with N(0,1) values), where the two bf16 roundings of the arithmetic (the weights, with the e4m3 scale folded in,
    and the output itself, 2^-9 relative each) already exceed 1e-2 absolute; the element-wise bound is therefore
    1e-2 + 2^-8 |ref| here, as for the prefill.  The row-relative and log-sum-exp bounds are the usual ones."""
    import paper_2507_01663_amd as ra
    from gpu_util import compare
    ulp = 2.0 ** -8
    d = {"self-planned": dec, "schedule kernels": dec_sched, "few waves": dec_few_waves}[which]
    rng = np.random.default_rng({"self-planned": 101, "schedule kernels": 202, "few waves": 303}[which])
    for case in range(10):
        Hkv = int(rng.choice([1, 2, 4, 8]))
        G = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 16]))
        D = int(rng.choice([64, 128]))
        ngroups, R = int(rng.integers(1, 9)), int(rng.integers(1, 13))
        prompts = rng.choice([0, 1, 15, 16, 17, 40, 64, 100, 333], size=ngroups)
        kind = rng.integers(0, 4, size=ngroups * R)
        resp = np.where(kind == 0, 0, np.where(kind == 1, rng.integers(1, 4, size=ngroups * R),
                        np.where(kind == 2, rng.integers(4, 200, size=ngroups * R), rng.integers(200, 2500, size=ngroups * R))))
        kv = "fp8_e4m3" if rng.integers(0, 3) == 0 else "bf16"
        p = workload.build_problem("random", Hkv * G, Hkv, D, prompts, R, resp, kv_dtype=kv, seed=1000 + case)
        if rng.integers(0, 2):                              # group ids need not be contiguous in b; some opt out
            perm = rng.permutation(p.B)
            for name in ("q", "block_table", "seq_lens", "seq_group"):
                setattr(p, name, np.ascontiguousarray(getattr(p, name)[perm]))
            p.seq_group[rng.integers(0, p.B)] = -1
        what = "%s case %d: Hq %d Hkv %d D %d groups %d x %d %s" % (which, case, Hkv * G, Hkv, D, ngroups, R, kv)
        log(what)
        ref = oracle.decode(p)
        compare(*run(d, p).results(), *ref, what, abs_rel=ulp)
        compare(*run(d, p, flags=ra.RA_FLAG_REUSE_SCHEDULE).results(), *ref, what + ", schedule reused", abs_rel=ulp)
        compare(*run(d, p, use_hint=False).results(), *ref, what + ", no hint", abs_rel=ulp)


@pytest.mark.parametrize("which", ["self-planned", "schedule kernels", "few waves"])
def test_reused_schedule_gives_the_same_bytes(dec, dec_sched, dec_few_waves, which):
    """A call that reuses the schedule (RA_FLAG_REUSE_SCHEDULE) streams exactly the spans of the call that made it:
    the same problem with and without the flag must give the same bytes, whether the schedule came from the schedule
    kernels, from attention waves that kept their lists, or from waves whose spans did not fit one list (those plan
    again).  bf16 and e4m3 pools; after a call on another batch the flag must not be used, and is not here."""
    import paper_2507_01663_amd as ra
    d = {"self-planned": dec, "schedule kernels": dec_sched, "few waves": dec_few_waves}[which]
    cases = [workload.make_problem("mid7b", seed=2), workload.make_problem("mid32b", seed=2, kv_dtype="fp8_e4m3"),
             workload.make_problem("grpo7b", seed=1)]
    if which == "few waves":
        rng = np.random.default_rng(159)
        resp = rng.integers(1, 3, size=6 * 70)
        resp[::70] = 111000
        cases.append(workload.build_problem("fragments", 4, 4, 128, [16] * 6, 70, resp, seed=31))
    for p in cases:
        plain = run(d, p)
        again = run(d, p, flags=ra.RA_FLAG_REUSE_SCHEDULE)
        third = run(d, p, flags=ra.RA_FLAG_REUSE_SCHEDULE)
        torch.cuda.synchronize()
        for other in (again, third):
            assert torch.equal(plain.out.view(torch.int16), other.out.view(torch.int16)) and torch.equal(plain.lse, other.lse)
        assert bool(torch.isfinite(plain.lse[torch.from_numpy(p.seq_lens > 0).to(plain.lse.device)]).all())


def test_wave_weights_move_work_not_results(dec):
    """The shares of the page stream that the attention workgroups get can be set per workgroup; any weights give the
    same answer within tolerance, and the same weights the same bytes."""
    import paper_2507_01663_amd as ra
    from gpu_util import compare
    p = workload.make_problem("mid7b", seed=4)
    ref = oracle.decode(p)
    n = ra.rollout_attn_wave_count(dec.ctx, ra.RA_KV_BF16, p.D)
    assert n > 0 and n % 8 == 0
    rng = np.random.default_rng(8)
    first = None
    try:
        for w in (rng.integers(700, 1401, size=n), rng.integers(700, 1401, size=n), np.full(n, 1000)):
            ra.rollout_attn_set_wave_weights(dec.ctx, w, ra.RA_KV_BF16, p.D)
            dp = run(dec, p)
            compare(*dp.results(), *ref, "random wave weights")
            dp2 = run(dec, p)
            torch.cuda.synchronize()
            assert torch.equal(dp.out.view(torch.int16), dp2.out.view(torch.int16)) and torch.equal(dp.lse, dp2.lse)
        with pytest.raises(ra.RolloutAttnError):
            ra.rollout_attn_set_wave_weights(dec.ctx, np.full(n - 1, 1000), ra.RA_KV_BF16, p.D)
    finally:
        ra.rollout_attn_set_wave_weights(dec.ctx, np.full(n, 1000), ra.RA_KV_BF16, p.D)
