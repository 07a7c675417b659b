"""Invariants of the schedule (the kernels that cut the page stream into spans and write every span's work
list), read back from the workspace after rollout_attn_debug_schedule: every page of every (work row, kv head)
item lies in exactly one span's list, lists are in stream order, records stay inside their tables, and the
merge descriptors name exactly the spans that hold an item's pages."""
import numpy as np
import pytest
import torch

import paper_2507_01663_amd as ra
import workload
from gpu_util import DeviceProblem

pytestmark = pytest.mark.gpu


def read_schedule(dec, dp):
    info, ws = dec.schedule(dp.c)
    torch.cuda.synchronize()
    raw = ws.cpu().numpy()
    hdr = raw[info.header_offset:info.header_offset + 64].view(np.int32)
    rec = raw[info.work_list_offset:].view(np.int32)
    p = dp.p
    md = raw[info.merge_desc_offset:info.merge_desc_offset + p.B * p.Hkv * 32].view(np.int32).reshape(p.B * p.Hkv, 2, 4)
    return info, hdr, rec, md


def check_schedule(dec, p, use_hint=True, label=""):
    dp = DeviceProblem(p, use_hint=use_hint)
    info, hdr, rec, md = read_schedule(dec, dp)
    nspans, nPR = int(hdr[7]), int(hdr[3])
    assert nspans == info.waves and int(hdr[2]) == p.B + nPR
    G = p.Hq // p.Hkv
    max_pages = p.block_table.shape[1]
    npages = (p.seq_lens.astype(np.int64) + 15) // 16
    nchunks = rec.size // 64
    own, shared = {}, {}          # item -> list of (span, lo, hi)
    for c in range(nspans):
        ch, hops = c, 0
        while ch >= 0:
            h = rec[ch * 64:ch * 64 + 64]
            n, nxt = int(h[0]), int(h[1])
            assert 0 <= n <= info.segments_per_chunk, (label, c, ch, n)
            assert nxt == -1 or nspans <= nxt < nchunks, (label, c, nxt)
            assert nxt == -1 or n == info.segments_per_chunk
            for j in range(n):
                idx, lo, hi, lim, where, who, nrows, slot = (int(x) for x in h[8 * (1 + j):8 * (2 + j)])
                kvh, is_shared = where & 0xffff, where >> 16
                assert 0 <= lo < hi and 0 <= kvh < p.Hkv and is_shared in (0, 1), (label, c, j)
                if not is_shared:
                    b = who
                    assert 0 <= b < p.B and nrows == G
                    skip = idx - b * max_pages
                    assert 0 <= skip and skip + hi <= npages[b], (label, "own pages past the sequence", b, skip, hi, npages[b])
                    assert lo * 16 < lim <= hi * 16 and lim <= p.seq_lens[b] - 16 * skip
                    assert slot == b * p.Hkv + kvh + c
                    own.setdefault((b, kvh), []).append((c, lo, hi, skip))
                else:
                    assert 0 <= idx and idx + hi <= p.prefix_pages.size and lim == 16 * hi, (label, "shared pages past the list")
                    assert 0 < nrows <= (64 if p.kv_dtype == "bf16" else 32) and nrows % G == 0 and 0 <= who and who + nrows // G <= p.B
                    row = (slot - c - kvh) // p.Hkv
                    assert 0 <= row < nPR and slot == row * p.Hkv + kvh + c
                    shared.setdefault((row, kvh), []).append((c, lo, hi, idx))
            ch = nxt
            hops += 1
            assert hops < 10000
    # every sequence's own pages, once and in order
    for b in range(p.B):
        for kvh in range(p.Hkv):
            pieces = own.get((b, kvh), [])
            d = md[b * p.Hkv + kvh]
            if not pieces:
                assert d[0, 1] > d[0, 2], (label, "descriptor names spans for an item without pages", b, kvh)
                continue
            skip = pieces[0][3]
            assert all(x[3] == skip for x in pieces)
            assert [x[0] for x in pieces] == sorted(x[0] for x in pieces)
            assert pieces[0][1] == 0 and pieces[-1][2] == npages[b] - skip, (label, b, kvh, pieces, npages[b], skip)
            for (c0, l0, h0, _), (c1, l1, h1, _) in zip(pieces, pieces[1:]):
                assert h0 == l1 and c0 < c1
            assert d[0, 0] == npages[b] - skip
            assert list(range(int(d[0, 1]), int(d[0, 2]) + 1)) == [x[0] for x in pieces], (label, "merge descriptor", b, kvh)
    # every shared row's pages, once and in order; sequences covered by shared rows skip exactly those pages
    starts = set(int(x) for x in p.prefix_page_offsets[:-1])
    for (row, kvh), pieces in shared.items():
        idx = pieces[0][3]
        assert idx in starts and all(x[3] == idx for x in pieces)
        g = int(np.searchsorted(p.prefix_page_offsets, idx, side="right") - 1)
        while p.prefix_page_offsets[g + 1] == idx:   # skip groups without shared pages that start at the same offset
            g += 1
        assert pieces[0][1] == 0 and pieces[-1][2] == p.prefix_page_offsets[g + 1] - idx
        for (c0, l0, h0, _), (c1, l1, h1, _) in zip(pieces, pieces[1:]):
            assert h0 == l1 and c0 < c1
    for b in range(p.B):
        for kvh in range(p.Hkv):
            d = md[b * p.Hkv + kvh, 1]
            skip = own[(b, kvh)][0][3] if (b, kvh) in own else None
            if d[1] <= d[2]:     # uses the shared pass
                assert use_hint and p.seq_group[b] >= 0
                g = int(p.seq_group[b])
                np_g = int(p.prefix_page_offsets[g + 1] - p.prefix_page_offsets[g])
                assert d[0] == np_g and (skip is None or skip == np_g)
            else:
                assert skip in (None, 0)
    return nspans


@pytest.fixture(scope="module")
def dec():
    d = ra.Decoder(0)
    yield d
    d.close()


@pytest.mark.parametrize("name", ["tiny", "mid7b", "mid32b", "mid72b", "grpo7b", "tail32b", "stream72b"])
def test_schedule_of_the_configurations(dec, name):
    # (the schedule reads lengths, groups and prefix offsets only: the two largest configurations get one dummy page)
    big = name in ("tail32b", "stream72b")
    p = workload.make_problem(name, seed=1, make_values=not big)
    if big:
        p.q = np.zeros((p.B, p.Hq, p.D), dtype=np.uint16)
        p.k_pool = p.v_pool = np.zeros((1, p.Hkv, 16, p.D), dtype=np.uint16)
    check_schedule(dec, p, True, name)
    check_schedule(dec, p, False, name + " (no hint)")


def test_schedule_of_random_batches(dec):
    rng = np.random.default_rng(123)
    for trial in range(25):
        Hkv = int(rng.choice([1, 2, 4, 8]))
        G = int(rng.choice([1, 2, 5, 7, 8, 16]))
        ngroups = int(rng.integers(1, 12))
        R = int(rng.integers(1, 20))
        prompts = rng.choice([0, 16, 17, 48, 200], size=ngroups)
        kind = trial % 3
        hi = [40, 600, 3000][kind]
        resp = rng.integers(0, hi, size=ngroups * R)
        resp[rng.random(resp.size) < 0.15] = 0
        p = workload.build_problem("rand%d" % trial, Hkv * G, Hkv, 64, prompts, R, resp, seed=trial, make_values=False)
        if trial % 4 == 0:      # some members shorter than their group's prefix, some ungrouped
            p.seq_lens = np.array(p.seq_lens, copy=True)
            p.seq_group = np.array(p.seq_group, copy=True)
            p.seq_lens[::5] = np.minimum(p.seq_lens[::5], 7)
            p.seq_group[1::7] = -1
        # the schedule reads lengths, groups and prefix offsets only: one dummy page stands for the pools
        p.q = np.zeros((p.B, p.Hq, p.D), dtype=np.uint16)
        p.k_pool = p.v_pool = np.zeros((1, Hkv, 16, 64), dtype=np.uint16)
        check_schedule(dec, p, True, "random %d" % trial)
