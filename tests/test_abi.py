"""CPU-side checks of the C ABI: the library loads, exports every symbol the header declares, and the
host-only argument checks return the documented status codes (no compute calls, no GPU needed)."""
import ctypes
import os
import re

import pytest

import paper_2507_01663_amd as ra

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "rollout_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rollout_attn_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ra.load_library()
    names = declared_symbols()
    assert len(names) == 20, names
    for n in names:
        assert getattr(lib, n) is not None
    assert ra.rollout_attn_abi_version() == 1


def test_struct_layout_matches_header_size():
    # 7 int32 (28) + pad to 8 -> 32; 3 ptr; 3 int64; int32 + pad; 2 ptr; 2 ptr; int32 + pad; 3 ptr; float + pad; 2 ptr; u32 + pad
    assert ctypes.sizeof(ra.ra_problem) == 32 + 24 + 24 + 8 + 16 + 16 + 8 + 24 + 8 + 16 + 8


def good_problem():
    p = ra.ra_problem()
    p.B, p.Hq, p.Hkv, p.D, p.page_size, p.num_pages, p.max_pages_per_seq = 4, 8, 2, 128, 16, 100, 10
    for f in ("q", "k_pool", "v_pool", "block_table", "seq_lens", "out", "lse"):
        setattr(p, f, 0x1000)           # never dereferenced by the host-side check
    p.kv_stride_page, p.kv_stride_head, p.kv_stride_token = 2 * 16 * 128, 16 * 128, 128
    p.softmax_scale = 0.1
    return p


def test_check_problem_status_codes():
    assert ra.rollout_attn_check_problem(good_problem())[0] == ra.RA_OK
    assert ra.rollout_attn_check_problem(None)[0] == ra.RA_ERR_INVALID_ARG
    cases = [
        (dict(Hq=7), ra.RA_ERR_INVALID_ARG, "multiple"),
        (dict(B=-1), ra.RA_ERR_INVALID_ARG, "dimension"),
        (dict(q=None), ra.RA_ERR_INVALID_ARG, "pointer"),
        (dict(lse=None), ra.RA_ERR_INVALID_ARG, "pointer"),
        (dict(kv_dtype=3), ra.RA_ERR_INVALID_ARG, "kv_dtype"),
        (dict(flags=64), ra.RA_ERR_INVALID_ARG, "flags"),
        (dict(softmax_scale=float("nan")), ra.RA_ERR_INVALID_ARG, "finite"),
        (dict(kv_stride_token=64), ra.RA_ERR_INVALID_ARG, "stride"),
        (dict(kv_stride_head=16 * 128 + 4), ra.RA_ERR_INVALID_ARG, "16 bytes"),
        (dict(k_pool=0x1004), ra.RA_ERR_INVALID_ARG, "aligned"),
        (dict(num_groups=2), ra.RA_ERR_INVALID_ARG, "num_groups"),
        (dict(page_size=32), ra.RA_ERR_UNSUPPORTED, "page_size"),
        (dict(D=96), ra.RA_ERR_UNSUPPORTED, "D="),
        (dict(Hq=64, Hkv=2), ra.RA_ERR_UNSUPPORTED, "Hq/Hkv"),
    ]
    for change, status, word in cases:
        p = good_problem()
        for k, v in change.items():
            setattr(p, k, v)
        st, msg = ra.rollout_attn_check_problem(p)
        assert st == status, (change, st, msg)
        assert word in msg, (change, msg)
    assert ra.rollout_attn_last_error(None) != ""
    # B == 0 is a valid, empty problem even without pointers
    p = ra.ra_problem()
    p.Hq, p.Hkv, p.D, p.page_size = 8, 2, 128, 16
    assert ra.rollout_attn_check_problem(p)[0] == ra.RA_OK


def good_prefill():
    p = ra.ra_prefill()
    p.num_prompts, p.total_tokens, p.max_prompt_len = 3, 700, 400
    p.Hq, p.Hkv, p.D = 28, 4, 128
    p.q, p.k, p.v, p.cu_seqlens = 0x10000, 0x20000, 0x30000, 0x40000
    p.softmax_scale = 0.1
    p.out, p.lse = 0x50000, 0x60000
    return p


def with_cache_write(p, fp8=False):
    p.k_pool, p.v_pool = 0x70000, 0x80000
    p.page_size, p.num_pages = 16, 64
    p.kv_stride_token, p.kv_stride_head, p.kv_stride_page = 128, 16 * 128, 4 * 16 * 128
    p.kv_dtype = ra.RA_KV_FP8_E4M3 if fp8 else ra.RA_KV_BF16
    if fp8:
        p.k_scale, p.v_scale = 0x90000, 0xA0000
    p.page_offsets, p.pages = 0xB0000, 0xC0000
    return p


def test_check_prefill_status_codes():
    assert ra.rollout_attn_check_prefill(good_prefill()) == (ra.RA_OK, "")
    assert ra.rollout_attn_check_prefill(with_cache_write(good_prefill())) == (ra.RA_OK, "")
    assert ra.rollout_attn_check_prefill(with_cache_write(good_prefill(), fp8=True)) == (ra.RA_OK, "")
    assert ra.rollout_attn_check_prefill(None)[0] == ra.RA_ERR_INVALID_ARG
    plain = [
        (dict(Hq=7), ra.RA_ERR_INVALID_ARG, "multiple"),
        (dict(num_prompts=-1), ra.RA_ERR_INVALID_ARG, "dimension"),
        (dict(max_prompt_len=-5), ra.RA_ERR_INVALID_ARG, "dimension"),
        (dict(Hkv=0), ra.RA_ERR_INVALID_ARG, "dimension"),
        (dict(q=None), ra.RA_ERR_INVALID_ARG, "pointer"),
        (dict(cu_seqlens=None), ra.RA_ERR_INVALID_ARG, "pointer"),
        (dict(lse=None), ra.RA_ERR_INVALID_ARG, "pointer"),
        (dict(k=0x20008), ra.RA_ERR_INVALID_ARG, "aligned"),
        (dict(lse=0x60002), ra.RA_ERR_INVALID_ARG, "aligned"),
        (dict(softmax_scale=float("inf")), ra.RA_ERR_INVALID_ARG, "finite"),
        (dict(softmax_scale=-1.0), ra.RA_ERR_INVALID_ARG, "positive"),
        (dict(D=96), ra.RA_ERR_UNSUPPORTED, "D="),
        (dict(total_tokens=2 ** 31 - 1, Hq=1024, Hkv=1024), ra.RA_ERR_UNSUPPORTED, "too large"),
    ]
    cache = [
        (dict(kv_dtype=3), ra.RA_ERR_INVALID_ARG, "kv_dtype"),
        (dict(page_size=32), ra.RA_ERR_UNSUPPORTED, "page_size"),
        (dict(v_pool=None), ra.RA_ERR_INVALID_ARG, "v_pool"),
        (dict(pages=None), ra.RA_ERR_INVALID_ARG, "pages"),
        (dict(num_pages=-1), ra.RA_ERR_INVALID_ARG, "num_pages"),
        (dict(kv_stride_token=64), ra.RA_ERR_INVALID_ARG, "stride"),
        (dict(kv_stride_page=-16), ra.RA_ERR_INVALID_ARG, "stride"),
        (dict(kv_stride_head=16 * 128 + 4), ra.RA_ERR_INVALID_ARG, "16 bytes"),
        (dict(kv_stride_token=2 ** 27), ra.RA_ERR_UNSUPPORTED, "too large"),
        (dict(k_pool=0x70004), ra.RA_ERR_INVALID_ARG, "aligned"),
    ]
    for base, cases in ((good_prefill, plain), (lambda: with_cache_write(good_prefill()), cache)):
        for change, status, word in cases:
            p = base()
            for k, v in change.items():
                setattr(p, k, v)
            st, msg = ra.rollout_attn_check_prefill(p)
            assert st == status, (change, st, msg)
            assert word in msg, (change, msg)
    p = with_cache_write(good_prefill(), fp8=True)
    p.v_scale = None
    st, msg = ra.rollout_attn_check_prefill(p)
    assert st == ra.RA_ERR_INVALID_ARG and "scale" in msg
    # without a cache write the pool fields are not looked at
    p = good_prefill()
    p.page_size, p.kv_dtype, p.kv_stride_token = 5, 9, -3
    assert ra.rollout_attn_check_prefill(p)[0] == ra.RA_OK
    # an empty batch is valid even without pointers
    p = ra.ra_prefill()
    p.Hq, p.Hkv, p.D, p.softmax_scale = 8, 2, 64, 0.125
    assert ra.rollout_attn_check_prefill(p)[0] == ra.RA_OK


def test_workspace_size_is_a_function_of_the_shape():
    p = good_problem()
    a = ra.rollout_attn_workspace_size(None, p)
    p.B = 8
    b = ra.rollout_attn_workspace_size(None, p)
    p.num_groups = 2
    c = ra.rollout_attn_workspace_size(None, p)
    assert 0 < a < b < c and a % 256 == 0
    p.D = 100
    with pytest.raises(ra.RolloutAttnError) as e:
        ra.rollout_attn_workspace_size(None, p)
    assert e.value.status == ra.RA_ERR_UNSUPPORTED
    p.D, p.Hq = 128, 7
    with pytest.raises(ra.RolloutAttnError) as e:
        ra.rollout_attn_workspace_size(None, p)
    assert e.value.status == ra.RA_ERR_INVALID_ARG


def test_decode_without_context_is_rejected():
    with pytest.raises(ra.RolloutAttnError) as e:
        ra.rollout_attn_decode(None, good_problem(), None, 0, None)
    assert e.value.status == ra.RA_ERR_INVALID_ARG


def test_create_without_a_gpu_reports_device_error(have_gpu):
    if have_gpu:
        pytest.skip("a GPU is present")
    with pytest.raises(ra.RolloutAttnError) as e:
        ra.rollout_attn_create(0)
    assert e.value.status == ra.RA_ERR_DEVICE
