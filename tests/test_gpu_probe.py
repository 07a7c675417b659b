"""The streaming probes (measurement aids of bench.py): they run, read what they say they read, end, and reject bad
arguments on the host."""
import ctypes

import pytest
import torch

import paper_2507_01663_amd as ra

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dec():
    ra.load_library()
    d = ra.Decoder(0)
    yield d
    d.close()


def test_probes_run_and_report_their_bytes(dec):
    buf = torch.zeros(1 << 26, dtype=torch.uint8, device="cuda:0")
    ptr = ctypes.c_void_p(buf.data_ptr())
    waves = ra.rollout_attn_wave_count(dec.ctx, ra.RA_KV_BF16, 128)
    for scattered in (0, 1, 2, 3):         # bit 0: scattered places; bit 1: ordinary loads instead of streaming ones
        for granule in (1024, 4096, 16384):
            assert ra.rollout_attn_debug_stream(dec.ctx, ptr, buf.numel(), granule, scattered, 5) == waves * 5 * 16384
    # static part of 3 entries, the other 2 per wave as tickets of 4 entries (the last chunk rounded up), twice in a
    # row (the counter starts from zero every time), then with nothing static at all
    n_tail = -(-waves * 2 // 4)
    for _ in range(2):
        assert ra.rollout_attn_debug_stream_tail(dec.ctx, ptr, buf.numel(), 5, 3, 4) == (waves * 3 + n_tail * 4) * 16384
    assert ra.rollout_attn_debug_stream_tail(dec.ctx, ptr, buf.numel(), 2, 0, 1) == waves * 2 * 16384
    torch.cuda.synchronize()


def test_probes_reject_bad_arguments(dec):
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda:0")
    ptr = ctypes.c_void_p(buf.data_ptr())
    bad = [lambda: ra.rollout_attn_debug_stream(dec.ctx, ptr, buf.numel() - 16, 4096, 1, 4),       # not a power of two
           lambda: ra.rollout_attn_debug_stream(dec.ctx, ptr, buf.numel(), 3000, 1, 4),
           lambda: ra.rollout_attn_debug_stream(dec.ctx, ptr, buf.numel(), 4096, 1, 0),
           lambda: ra.rollout_attn_debug_stream(dec.ctx, None, buf.numel(), 4096, 1, 4),
           lambda: ra.rollout_attn_debug_stream_tail(dec.ctx, ptr, buf.numel(), 4, 4, 2),          # nothing left for tickets
           lambda: ra.rollout_attn_debug_stream_tail(dec.ctx, ptr, buf.numel(), 4, -1, 2),
           lambda: ra.rollout_attn_debug_stream_tail(dec.ctx, ptr, buf.numel(), 4, 2, 0),
           lambda: ra.rollout_attn_debug_stream_tail(dec.ctx, ctypes.c_void_p(buf.data_ptr() + 4), buf.numel(), 4, 2, 2)]
    for f in bad:
        with pytest.raises(ra.RolloutAttnError) as e:
            f()
        assert e.value.status == ra.RA_ERR_INVALID_ARG
    torch.cuda.synchronize()
