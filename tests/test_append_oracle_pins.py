"""Pins for the KV-append oracle (CPU only).  The paper defines no append (it is the write that auto-regressive
generation, Sec. 2.1.1, performs before each decode step's attention), so the oracle's own definition is pinned
by what mathematics and independent routines fix: the E4M3 encoder against the format's table, torch's cast and
the input generator's encoder; the bf16 write against a numpy fancy-index write; the quantised write against the
generator's page quantiser, error bounds and invariants."""
import copy

import numpy as np
import pytest
import torch

import oracle
import workload
from workload.gen import build_problem, bf16_bits_to_f32, f32_to_bf16_bits


def writable(p):
    p = copy.copy(p)
    p.k_pool = np.array(p.k_pool, copy=True)
    p.v_pool = np.array(p.v_pool, copy=True)
    if p.kv_dtype == "fp8_e4m3":
        p.k_scale = np.array(p.k_scale, copy=True)
        p.v_scale = np.array(p.v_scale, copy=True)
    p.seq_lens = np.array(p.seq_lens, copy=True)
    return p


def small(kvd, lens, seed=3, Hkv=2, D=64):
    lens = np.asarray(lens, dtype=np.int64)
    return writable(build_problem("append", 2 * Hkv, Hkv, D, np.zeros(len(lens), dtype=np.int64), 1, lens, kv_dtype=kvd,
                                  seed=seed, slack=2.0))


def with_room(p):
    """One more table column, and a free page wherever the next token starts a page."""
    bt = np.full((p.B, p.block_table.shape[1] + 1), -1, dtype=np.int32)
    bt[:, :-1] = p.block_table
    free = iter(sorted(set(range(p.num_pages)) - set(bt[bt >= 0].tolist())))
    for b in range(p.B):
        if bt[b, p.seq_lens[b] // 16] < 0:
            bt[b, p.seq_lens[b] // 16] = next(free)
    p.block_table = bt
    return p


def new_rows(B, Hkv, D, seed, scale=1.0):
    r = np.random.default_rng(seed)
    return f32_to_bf16_bits((r.standard_normal((B, Hkv, D)) * scale).astype(np.float32))


# ---- encoder ---------------------------------------------------------------------------------------------

def test_encoder_round_trips_every_code_and_rounds_to_nearest_even():
    tab = oracle.e4m3_decode_table()
    finite = np.array([c for c in range(256) if not np.isnan(tab[c]) and tab[c] != 0])
    np.testing.assert_array_equal(oracle.e4m3_encode(tab[finite].astype(np.float32)), finite)
    # midpoints between neighbours go to the even code (the one whose last mantissa bit is 0)
    pos = np.sort(tab[(tab >= 0) & ~np.isnan(tab)])
    pos = np.unique(pos)
    mids = ((pos[:-1] + pos[1:]) / 2).astype(np.float32)
    assert np.all(mids.astype(np.float64) == (pos[:-1] + pos[1:]) / 2)  # midpoints are binary32 values
    got = oracle.e4m3_encode(mids)
    lo_code = oracle.e4m3_encode(pos[:-1].astype(np.float32))
    hi_code = oracle.e4m3_encode(pos[1:].astype(np.float32))
    want = np.where(lo_code % 2 == 0, lo_code, hi_code)
    np.testing.assert_array_equal(got, want)
    # saturation, signs, NaN
    assert oracle.e4m3_encode(np.float32([448, 449, 1e30, np.inf])).tolist() == [0x7E] * 4
    assert oracle.e4m3_encode(np.float32([-448, -1e30, -np.inf])).tolist() == [0xFE] * 3
    assert oracle.e4m3_encode(np.float32([np.nan]))[0] == 0x7F


def test_encoder_agrees_with_torch_cast_and_with_the_generators_encoder():
    r = np.random.default_rng(0)
    y = np.concatenate([r.standard_normal(20000) * 100, r.standard_normal(20000), r.standard_normal(20000) * 1e-2,
                        r.uniform(-448, 448, 20000)]).astype(np.float32)
    y = y[np.abs(y) <= 448]
    mine = oracle.e4m3_encode(y)
    lib = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    tab = oracle.e4m3_decode_table()
    np.testing.assert_array_equal(tab[mine], tab[lib])          # (+0 and -0 compare equal)
    np.testing.assert_array_equal(tab[mine], tab[workload.e4m3_encode(y)])
    # nearest: no other code is closer
    err = np.abs(tab[mine] - y.astype(np.float64))
    finite = tab[~np.isnan(tab)]
    best = np.min(np.abs(finite[None, :] - y[:2000, None].astype(np.float64)), axis=1)
    np.testing.assert_array_equal(err[:2000], best)


# ---- bf16 ------------------------------------------------------------------------------------------------

def test_bf16_append_is_the_addressed_copy():
    p = small("bf16", [0, 1, 15, 16, 17, 40])
    k0, v0 = p.k_pool.copy(), p.v_pool.copy()
    kn, vn = new_rows(p.B, p.Hkv, p.D, 1), new_rows(p.B, p.Hkv, p.D, 2)
    with_room(p)
    assert oracle.append(p, kn, vn) == 0
    ek, ev = k0.copy(), v0.copy()
    pg = p.block_table[np.arange(p.B), p.seq_lens // 16]
    ek[pg, :, p.seq_lens % 16, :] = kn
    ev[pg, :, p.seq_lens % 16, :] = vn
    np.testing.assert_array_equal(p.k_pool, ek)
    np.testing.assert_array_equal(p.v_pool, ev)


def test_out_of_range_sequences_are_skipped_and_nothing_else_is_touched():
    p = small("bf16", [5, 20, 33])
    p.block_table = np.array(p.block_table, copy=True)
    cap = p.block_table.shape[1] * 16
    p.seq_lens[0] = cap            # no room in the table row
    p.seq_lens[1] = -3
    p.block_table[2, 33 // 16] = p.num_pages   # page id out of range
    k0, v0 = p.k_pool.copy(), p.v_pool.copy()
    assert oracle.append(p, new_rows(p.B, p.Hkv, p.D, 1), new_rows(p.B, p.Hkv, p.D, 2)) == 3
    np.testing.assert_array_equal(p.k_pool, k0)
    np.testing.assert_array_equal(p.v_pool, v0)


# ---- e4m3 ------------------------------------------------------------------------------------------------

def fresh_fp8(lens, seed=5):
    return with_room(small("fp8_e4m3", lens, seed=seed))


def test_fp8_first_slot_of_a_page_matches_the_generators_page_quantiser():
    p = fresh_fp8([0, 16, 32])
    kn, vn = new_rows(p.B, p.Hkv, p.D, 7), new_rows(p.B, p.Hkv, p.D, 8, scale=0.01)
    kn[1, 0, :] = 0                                   # an all-zero row: scale 1, codes 0
    assert oracle.append(p, kn, vn) == 0
    tab = oracle.e4m3_decode_table()
    for b in range(p.B):
        pg = p.block_table[b, p.seq_lens[b] // 16]
        for new, pool, scale in ((kn, p.k_pool, p.k_scale), (vn, p.v_pool, p.v_scale)):
            for h in range(p.Hkv):
                x = bf16_bits_to_f32(new[b, h])
                amax = np.abs(x).max()
                want_scale = np.float32(amax / np.float32(448)) if amax > 0 else np.float32(1)
                assert scale[pg, h] == want_scale
                codes = pool[pg, h, 0]
                # a tile holding this one row and zeros quantises to the same scale and codes
                tile = np.zeros((1, 16 * p.D), dtype=np.uint16)
                tile[0, :p.D] = new[b, h]
                gc, gs = workload.gen._quantise_tiles(tile)
                assert gs[0] == want_scale
                np.testing.assert_array_equal(tab[codes], tab[gc[0, :p.D]])
                # and the error is at most half a step of the code's binade
                err = np.abs(tab[codes] * float(want_scale) - x.astype(np.float64))
                step = np.where(np.abs(tab[codes]) < 2.0 ** -6, 2.0 ** -9, 2.0 ** (np.floor(np.log2(np.maximum(np.abs(tab[codes]), 1e-30))) - 3))
                assert np.all(err <= 0.5 * step * float(want_scale) * (1 + 1e-6) + 1e-12)


def test_fp8_smaller_row_keeps_the_scale_and_the_stored_codes():
    p = fresh_fp8([3, 21])
    before_k, before_ks = p.k_pool.copy(), p.k_scale.copy()
    kn = new_rows(p.B, p.Hkv, p.D, 9, scale=1e-3)
    vn = new_rows(p.B, p.Hkv, p.D, 10, scale=1e-3)
    assert oracle.append(p, kn, vn) == 0
    np.testing.assert_array_equal(p.k_scale, before_ks)
    tab = oracle.e4m3_decode_table()
    for b in range(p.B):
        pg, s = p.block_table[b, p.seq_lens[b] // 16], p.seq_lens[b] % 16
        np.testing.assert_array_equal(p.k_pool[pg, :, :s], before_k[pg, :, :s])
        for h in range(p.Hkv):
            x = bf16_bits_to_f32(kn[b, h])
            want = oracle.e4m3_encode((x / before_ks[pg, h]).astype(np.float32))
            np.testing.assert_array_equal(tab[p.k_pool[pg, h, s]], tab[want])
    # every other page is untouched
    touched = set(int(p.block_table[b, p.seq_lens[b] // 16]) for b in range(p.B))
    others = [g for g in range(p.num_pages) if g not in touched]
    np.testing.assert_array_equal(p.k_pool[others], before_k[others])


def test_fp8_larger_row_rescales_the_page():
    p = fresh_fp8([5, 30])
    tab = oracle.e4m3_decode_table()
    before_k, before_ks = p.k_pool.copy(), p.k_scale.copy()
    kn = new_rows(p.B, p.Hkv, p.D, 11, scale=50.0)     # far above the stored rows (N(0,1) data)
    vn = new_rows(p.B, p.Hkv, p.D, 12, scale=50.0)
    assert oracle.append(p, kn, vn) == 0
    for b in range(p.B):
        pg, s = p.block_table[b, p.seq_lens[b] // 16], p.seq_lens[b] % 16
        for h in range(p.Hkv):
            x = bf16_bits_to_f32(kn[b, h])
            new_scale = np.float32(np.abs(x).max() / np.float32(448))
            assert p.k_scale[pg, h] == new_scale and new_scale > before_ks[pg, h]
            # the new row uses the whole range, its absmax element maps to +-448
            assert np.abs(tab[p.k_pool[pg, h, s]]).max() == 448
            # stored rows: re-quantised from their dequantised values, binary32 throughout (numpy float32 ops)
            old_val = (tab[before_k[pg, h, :s]].astype(np.float32) * before_ks[pg, h]).astype(np.float32)
            want = oracle.e4m3_encode((old_val / new_scale).astype(np.float32))
            np.testing.assert_array_equal(tab[p.k_pool[pg, h, :s]], tab[want])
            # so each stays within half a (new, coarser) step of what it stood for
            now = tab[p.k_pool[pg, h, :s]] * float(new_scale)
            code_abs = np.abs(tab[p.k_pool[pg, h, :s]])
            step = np.where(code_abs < 2.0 ** -6, 2.0 ** -9, 2.0 ** (np.floor(np.log2(np.maximum(code_abs, 1e-30))) - 3))
            assert np.all(np.abs(now - old_val.astype(np.float64)) <= 0.5 * step * float(new_scale) * (1 + 1e-6) + 1e-12)
            # slots after the new one are not touched
            np.testing.assert_array_equal(p.k_pool[pg, h, s + 1:], before_k[pg, h, s + 1:])


def test_fp8_filling_a_page_token_by_token_then_attention_is_close_to_bf16_attention():
    """Sixteen appends fill a fresh page; the quantised cache then gives nearly the attention of the exact one
    (the oracle's attention is pinned elsewhere), and the scale is the running absmax / 448."""
    D, Hkv = 64, 2
    r = np.random.default_rng(4)
    rows_k = f32_to_bf16_bits(r.standard_normal((16, 1, Hkv, D)).astype(np.float32))
    rows_v = f32_to_bf16_bits(r.standard_normal((16, 1, Hkv, D)).astype(np.float32))
    p8 = fresh_fp8([0], seed=6)
    p16 = with_room(small("bf16", [0], seed=6))
    run_max = np.zeros(Hkv, dtype=np.float32)
    for t in range(16):
        assert oracle.append(p8, rows_k[t], rows_v[t]) == 0
        assert oracle.append(p16, rows_k[t], rows_v[t]) == 0
        p8.seq_lens[0] += 1
        p16.seq_lens[0] += 1
        run_max = np.maximum(run_max, np.abs(bf16_bits_to_f32(rows_k[t, 0])).max(axis=1))
        pg = p8.block_table[0, 0]
        np.testing.assert_array_equal(p8.k_scale[pg], run_max / np.float32(448))
    o8, l8 = oracle.decode(p8)
    o16, l16 = oracle.decode(p16)
    assert np.max(np.abs(o8 - o16)) < 0.1 and np.max(np.abs(l8 - l16)) < 0.1
