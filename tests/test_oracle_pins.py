"""Pins for the fp64 oracle: closed forms, invariants, brute force and library
routines.  The paper prints no worked numeric example for decode attention, so
every pin is mathematical.  Each is chosen so that a plausible mistake in the
oracle (dropped scale, wrong head mapping, page/slot swapped, K and V swapped,
missing max subtraction, wrong log base) fails at least one of them."""
import math

import numpy as np
import pytest
import scipy.special
import torch

import oracle
import workload
from workload import PAGE, bf16_bits_to_f32, f32_to_bf16_bits


def f64(bits):
    return bf16_bits_to_f32(bits).astype(np.float64)


def dense_reference(p, b, h):
    """Brute force: numpy fancy-index gather, then dense softmax(K q * scale) V."""
    G = p.Hq // p.Hkv
    kv = h // G
    L = int(p.seq_lens[b])
    t = np.arange(L)
    pages = p.block_table[b, t // PAGE]
    slots = t % PAGE
    if p.kv_dtype == "bf16":
        K = f64(p.k_pool[pages, kv, slots])
        V = f64(p.v_pool[pages, kv, slots])
    else:
        tab = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
        K = tab[p.k_pool[pages, kv, slots]] * p.k_scale[pages, kv].astype(np.float64)[:, None]
        V = tab[p.v_pool[pages, kv, slots]] * p.v_scale[pages, kv].astype(np.float64)[:, None]
    s = float(p.softmax_scale) * (K @ f64(p.q[b, h]))
    w = scipy.special.softmax(s)
    return w @ V, float(scipy.special.logsumexp(s)), w


def small(prompt_lens, R, resp_lens, Hq=4, Hkv=2, D=16, seed=0, **kw):
    return workload.build_problem("t", Hq, Hkv, D, prompt_lens, R, resp_lens, seed=seed, **kw)


@pytest.mark.parametrize("name,kvd", [("tiny", "bf16"), ("midd64", "bf16"), ("tiny", "fp8_e4m3"),
                                      ("mid7b", "bf16"), ("midd64", "fp8_e4m3")])
def test_matches_dense_brute_force(name, kvd):
    p = workload.make_problem(name, kv_dtype=kvd)
    out, lse = oracle.decode(p)
    rng = np.random.default_rng(1)
    rows = [(b, h) for b in range(p.B) for h in range(p.Hq)]
    if len(rows) > 64:
        rows = [rows[i] for i in rng.choice(len(rows), 64, replace=False)]
    for b, h in rows:
        ro, rl, _ = dense_reference(p, b, h)
        np.testing.assert_allclose(out[b, h], ro, rtol=1e-12, atol=1e-13)
        assert abs(lse[b, h] - rl) < 1e-12


def test_ragged_prompt_not_page_aligned():
    # prompt 20 tokens: one shared page, 4 prompt tokens spill into each member's own pages
    p = small([20, 7], 3, [0, 5, 40, 1, 0, 29])
    assert list(np.diff(p.prefix_page_offsets)) == [1, 0]
    out, lse = oracle.decode(p)
    for b in range(p.B):
        for h in range(p.Hq):
            ro, rl, _ = dense_reference(p, b, h)
            np.testing.assert_allclose(out[b, h], ro, rtol=1e-12, atol=1e-13)
            assert abs(lse[b, h] - rl) < 1e-12


def test_one_key_gives_v_and_score():
    p = small([0], 2, [1, 1], D=32)
    out, lse = oracle.decode(p)
    for b in range(2):
        pg = p.block_table[b, 0]
        for h in range(p.Hq):
            kv = h // 2
            np.testing.assert_array_equal(out[b, h], f64(p.v_pool[pg, kv, 0]))
            s = float(p.softmax_scale) * np.dot(f64(p.q[b, h]), f64(p.k_pool[pg, kv, 0]))
            assert abs(lse[b, h] - s) < 1e-13


def test_equal_scores_give_mean_of_v():
    p = small([16], 2, [21, 3])
    p.q[:] = 0                                   # every score is 0
    out, lse = oracle.decode(p)
    for b in range(p.B):
        L = int(p.seq_lens[b])
        for h in range(p.Hq):
            k, v, _ = oracle.gather(p, b, h // 2)
            np.testing.assert_allclose(out[b, h], f64(v).mean(axis=0), rtol=1e-13, atol=1e-14)
            assert abs(lse[b, h] - math.log(L)) < 1e-13
    # identical keys, non-zero query: lse = s + ln L
    p2 = small([0], 1, [37])
    p2.k_pool[:] = p2.k_pool[0, 0, 0]
    out2, lse2 = oracle.decode(p2)
    for h in range(p2.Hq):
        s = float(p2.softmax_scale) * np.dot(f64(p2.q[0, h]), f64(p2.k_pool[0, 0, 0]))
        _, v, _ = oracle.gather(p2, 0, h // 2)
        np.testing.assert_allclose(out2[0, h], f64(v).mean(axis=0), rtol=1e-12, atol=1e-13)
        assert abs(lse2[0, h] - (s + math.log(37))) < 1e-12


def test_two_keys_closed_form():
    p = small([0], 1, [2], D=32)
    out, lse = oracle.decode(p)
    pg = p.block_table[0, 0]
    for h in range(p.Hq):
        kv = h // 2
        q = f64(p.q[0, h])
        s1, s2 = (float(p.softmax_scale) * np.dot(q, f64(p.k_pool[pg, kv, i])) for i in (0, 1))
        sig = 1.0 / (1.0 + math.exp(s2 - s1))
        ref = sig * f64(p.v_pool[pg, kv, 0]) + (1 - sig) * f64(p.v_pool[pg, kv, 1])
        np.testing.assert_allclose(out[0, h], ref, rtol=1e-13, atol=1e-14)
        assert abs(lse[0, h] - np.logaddexp(s1, s2)) < 1e-13


def test_rows_of_p_sum_to_one():
    p = workload.make_problem("midd64")
    for b, h in [(0, 0), (3, 5), (11, 7)]:
        w, out, lse = oracle.probs(p, b, h)
        assert w.shape == (p.seq_lens[b],)
        assert (w >= 0).all() and abs(w.sum() - 1.0) < 1e-13
        _, _, wr = dense_reference(p, b, h)
        np.testing.assert_allclose(w, wr, rtol=1e-11, atol=1e-300)


def test_score_shift_invariance():
    # dimension 0 of every key is the constant 2; changing q[...,0] by a adds scale*2*a to every score
    p = small([16], 2, [30, 9], D=32)
    p.k_pool[..., 0] = f32_to_bf16_bits(np.float32(2.0))
    p.q[..., 0] = 0
    out0, lse0 = oracle.decode(p)
    p.q[..., 0] = f32_to_bf16_bits(np.float32(3.0))
    out1, lse1 = oracle.decode(p)
    np.testing.assert_allclose(out1, out0, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse1 - lse0, float(p.softmax_scale) * 6.0, rtol=0, atol=1e-12)


def test_large_scores_do_not_overflow():
    p = small([0], 1, [50], D=16, softmax_scale=40.0)
    out, lse = oracle.decode(p)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    assert np.abs(lse).max() > 80          # scores really are large
    for h in range(p.Hq):
        ro, rl, _ = dense_reference(p, 0, h)
        np.testing.assert_allclose(out[0, h], ro, rtol=1e-12, atol=1e-13)
        assert abs(lse[0, h] - rl) < 1e-10


def test_equal_length_batch_matches_library_sdpa():
    D, Hq, Hkv, L = 32, 6, 2, 45
    p = small([16, 16], 2, [L - 16] * 4, Hq=Hq, Hkv=Hkv, D=D)
    out, lse = oracle.decode(p)
    K = np.stack([np.stack([f64(oracle.gather(p, b, kv)[0]) for kv in range(Hkv)]) for b in range(p.B)])
    V = np.stack([np.stack([f64(oracle.gather(p, b, kv)[1]) for kv in range(Hkv)]) for b in range(p.B)])
    q = torch.from_numpy(f64(p.q)).unsqueeze(2)                       # [B,Hq,1,D]
    Kt = torch.from_numpy(K).repeat_interleave(Hq // Hkv, dim=1)      # [B,Hq,L,D]
    Vt = torch.from_numpy(V).repeat_interleave(Hq // Hkv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(q, Kt, Vt, scale=float(p.softmax_scale))
    np.testing.assert_allclose(out, ref.squeeze(2).numpy(), rtol=1e-11, atol=1e-12)
    s = float(p.softmax_scale) * torch.einsum("bhd,bhld->bhl", q.squeeze(2), Kt)
    np.testing.assert_allclose(lse, torch.logsumexp(s, dim=-1).numpy(), rtol=0, atol=1e-12)


def test_gqa_equals_replicated_mha():
    p = small([16], 2, [20, 3], Hq=6, Hkv=2, D=16)
    out, lse = oracle.decode(p)
    import copy
    m = copy.copy(p)
    m.Hkv = 6
    m.k_pool = np.repeat(p.k_pool, 3, axis=1)
    m.v_pool = np.repeat(p.v_pool, 3, axis=1)
    out2, lse2 = oracle.decode(m)
    np.testing.assert_array_equal(out, out2)
    np.testing.assert_array_equal(lse, lse2)


def test_page_permutation_invariance_is_bit_exact():
    p = workload.make_problem("midd64")
    out, lse = oracle.decode(p)
    perm = np.random.default_rng(5).permutation(p.num_pages)
    import copy
    m = copy.copy(p)
    inv = np.empty_like(perm)
    inv[perm] = np.arange(p.num_pages)
    m.k_pool = p.k_pool[perm]                   # new page i holds old page perm[i]
    m.v_pool = p.v_pool[perm]
    m.block_table = np.where(p.block_table >= 0, inv[np.maximum(p.block_table, 0)], -1).astype(np.int32)
    out2, lse2 = oracle.decode(m)
    np.testing.assert_array_equal(out, out2)
    np.testing.assert_array_equal(lse, lse2)


def test_gather_reads_the_addressed_page_and_slot():
    # every element encodes (page, kv head, slot); K and V differ in the top bit
    p = small([32], 2, [5, 40], Hq=4, Hkv=2, D=16)
    pg, kv, sl = np.meshgrid(np.arange(p.num_pages), np.arange(2), np.arange(PAGE), indexing="ij")
    code = (pg * 64 + kv * 32 + sl).astype(np.uint16)
    p.k_pool[:] = code[..., None]
    p.v_pool[:] = (code | 0x8000)[..., None]
    for b in range(p.B):
        for kvh in range(2):
            k, v, pages = oracle.gather(p, b, kvh)
            t = np.arange(p.seq_lens[b])
            want = p.block_table[b, t // PAGE] * 64 + kvh * 32 + t % PAGE
            np.testing.assert_array_equal(pages, p.block_table[b, t // PAGE])
            np.testing.assert_array_equal(k, np.broadcast_to(want[:, None], k.shape))
            np.testing.assert_array_equal(v, np.broadcast_to((want | 0x8000)[:, None], v.shape))


def test_merge_of_key_partitions_equals_whole():
    # whole sequence vs the same keys cut into three sequences (prompt pages, middle, rest)
    D, cut1, cut2, L = 16, 32, 80, 123
    whole = small([0], 1, [L], D=D, poison=False)
    out, lse = oracle.decode(whole)
    import copy
    parts = []
    for lo, hi in [(0, cut1), (cut1, cut2), (cut2, L)]:
        s = copy.copy(whole)
        s.block_table = whole.block_table[:, lo // PAGE:].copy()
        s.max_pages_per_seq = s.block_table.shape[1]
        s.seq_lens = np.array([hi - lo], dtype=np.int32)
        parts.append(oracle.decode(s))
    for h in range(whole.Hq):
        mo, ml = oracle.merge_partials(np.stack([po[0, h] for po, _ in parts]), np.array([pl[0, h] for _, pl in parts]))
        np.testing.assert_allclose(mo, out[0, h], rtol=1e-12, atol=1e-14)
        assert abs(ml - lse[0, h]) < 1e-13
    # an empty set does not change the result
    mo, ml = oracle.merge_partials(np.stack([out[0, 0], np.zeros(D)]), np.array([lse[0, 0], -np.inf]))
    np.testing.assert_allclose(mo, out[0, 0], rtol=1e-15)
    assert ml == lse[0, 0]


def test_empty_sequence():
    p = small([0], 2, [0, 3])
    out, lse = oracle.decode(p)
    assert (out[0] == 0).all() and np.isneginf(lse[0]).all()
    assert np.isfinite(lse[1]).all()


def test_row_subset_matches_full():
    p = workload.make_problem("midd64")
    out, lse = oracle.decode(p)
    rows = np.array([0, 17, 95, 40], dtype=np.int32)
    o2, l2 = oracle.decode(p, rows=rows)
    np.testing.assert_array_equal(o2, out.reshape(-1, p.D)[rows])
    np.testing.assert_array_equal(l2, lse.reshape(-1)[rows])


def test_out_of_range_page_is_an_error():
    p = small([0], 1, [20])
    p.block_table[0, 1] = p.num_pages
    with pytest.raises(ValueError):
        oracle.decode(p)


def test_poison_never_reaches_the_result():
    p = workload.make_problem("mid32b")
    assert (p.k_pool == workload.BF16_NAN).any()
    out, lse = oracle.decode(p)
    assert np.isfinite(out).all() and np.isfinite(lse).all()


# ---- e4m3 -------------------------------------------------------------------

def test_e4m3_table_matches_closed_form_and_library():
    tab = oracle.e4m3_decode_table()
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    for c in range(256):
        s, e, m = c >> 7, (c >> 3) & 15, c & 7
        if e == 15 and m == 7:
            assert math.isnan(tab[c]) and math.isnan(lib[c])
            continue
        want = (m / 8.0) * 2.0 ** -6 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7)
        want = -want if s else want
        assert tab[c] == want == lib[c]
    assert tab[0x7E] == 448.0 and tab[0x01] == 2.0 ** -9 and tab[0x08] == 2.0 ** -6


def test_e4m3_encode_is_nearest_even_and_saturates():
    tab = oracle.e4m3_decode_table()
    finite = np.array([c for c in range(256) if not math.isnan(tab[c])])
    # every representable value encodes to itself
    np.testing.assert_array_equal(tab[workload.e4m3_encode(tab[finite].astype(np.float32))], tab[finite])
    y = np.random.default_rng(0).standard_normal(20000).astype(np.float32) * np.float32(100.0)
    y = np.concatenate([y, np.float32([0.0, 1e-4, 2.0 ** -10, 3 * 2.0 ** -10, 447.9, 460.0, 1e6, -1e6, 17.0, 19.0])])
    dec = tab[workload.e4m3_encode(y)]
    pos = np.sort(tab[finite][tab[finite] >= 0])
    for yi, di in zip(y.astype(np.float64), dec):
        a = min(abs(yi), 448.0)
        best = np.min(np.abs(pos - a))
        assert abs(abs(di) - a) == best                     # nearest
        assert di == 0 or (di < 0) == (yi < 0)
    # ties go to the even mantissa: 17 is halfway between 16 and 18 -> 16; 19 -> 20
    assert tab[workload.e4m3_encode(np.float32([17.0, 19.0]))].tolist() == [16.0, 20.0]
    assert tab[workload.e4m3_encode(np.float32([3 * 2.0 ** -10]))][0] == 2 * 2.0 ** -9
    # torch's cast as a library cross-check (round to nearest even, in range)
    yy = np.clip(y, -448, 448)
    lib = torch.from_numpy(yy).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    mine = workload.e4m3_encode(yy)
    np.testing.assert_array_equal(tab[mine], tab[lib])


def test_fp8_pool_quantisation_error_bound():
    D = 64
    vals = workload.normal_bf16(64 * PAGE * D, 3, 7).reshape(64, PAGE * D)
    from workload.gen import _quantise_tiles
    codes, scale = _quantise_tiles(vals)
    x = f64(vals)
    tab = oracle.e4m3_decode_table()
    deq = tab[codes] * scale.astype(np.float64)[:, None]
    y = np.abs(x / scale.astype(np.float64)[:, None])
    e = np.maximum(np.floor(np.log2(np.maximum(y, 1e-300))), -6)
    half_ulp = 2.0 ** (e - 4)
    assert (np.abs(deq - x) <= scale[:, None] * half_ulp * (1 + 1e-6) + 1e-12).all()
    assert np.abs(tab[codes]).max() == 448.0                 # absmax maps to the largest code


# ---- workload recipes -------------------------------------------------------

def test_tiny_config_is_the_stated_one():
    p = workload.make_problem("tiny")
    assert (p.B, p.Hq, p.Hkv, p.D, p.page_size) == (4, 4, 2, 64, 16)
    assert p.seq_lens.tolist() == [17, 64, 100, 256]
    assert p.prefix_page_offsets.tolist() == [0, 1] and float(p.softmax_scale) == 0.125
    assert (p.block_table[:, 0] == p.prefix_pages[0]).all()


def test_grpo_shapes_and_algorithmic_bytes():
    p = workload.make_problem("grpo7b", make_values=False)
    assert (p.B, p.Hq, p.Hkv, p.D) == (256, 28, 4, 128)
    r = p.meta["resp_lens"]
    assert r.min() >= 0 and r.max() <= 3584 and (p.seq_lens == 512 + r).all()
    tok = 32 * 512 + int(r.sum())
    want = tok * 2048 + 2 * 256 * 28 * 128 * 2 + 4 * 256 * 28 + 4 * int(((p.seq_lens + 15) // 16).sum()) + 4 * 256
    assert p.algorithmic_bytes() == want
    assert p.algorithmic_bytes(share_prefix=False) == want + 7 * 32 * 512 * 2048
    # every member's row starts with its group's shared pages; no page is used twice otherwise
    for g in range(32):
        sh = p.prefix_pages[p.prefix_page_offsets[g]:p.prefix_page_offsets[g + 1]]
        assert len(sh) == 32
        for b in range(g * 8, g * 8 + 8):
            assert (p.block_table[b, :32] == sh).all()
    own = np.concatenate([p.block_table[b, 32:(p.seq_lens[b] + 15) // 16] for b in range(256)])
    allp = np.concatenate([own, p.prefix_pages])
    assert len(np.unique(allp)) == len(allp) and allp.max() < p.num_pages


def test_streaming_lengths_bookkeeping():
    cfg = workload.CONFIGS["mid72b"]
    prev = workload.response_lengths(cfg, 0, 0)
    resets = 0
    for s in range(1, 8):
        cur = workload.response_lengths(cfg, 0, s)
        grew = cur == prev + 1
        reset = cur == 0
        assert (grew | reset).all()
        resets += int((reset & ~grew).sum())
        prev = cur
    p0 = workload.make_problem("mid72b", step=0)
    p1 = workload.make_problem("mid72b", step=1, pool=(p0.k_pool, p0.v_pool, None, None), num_pages=p0.num_pages)
    assert p1.k_pool is p0.k_pool and not np.array_equal(p0.block_table[:, :4], p1.block_table[:, :4])


def test_generator_is_deterministic():
    a = workload.make_problem("midd64", seed=3)
    b = workload.make_problem("midd64", seed=3)
    c = workload.make_problem("midd64", seed=4)
    assert np.array_equal(a.k_pool, b.k_pool) and np.array_equal(a.block_table, b.block_table)
    assert not np.array_equal(a.q, c.q)


def test_frozen_tiny_fixture():
    """tests/golden/tiny_seed0.json was written by tests/golden/make_golden.py
    from the oracle alone; inputs and results must not drift."""
    import hashlib
    import json
    import os
    with open(os.path.join(os.path.dirname(__file__), "golden", "tiny_seed0.json")) as f:
        gold = json.load(f)
    for kvd in ("bf16", "fp8_e4m3"):
        p = workload.make_problem("tiny", seed=0, kv_dtype=kvd)
        h = hashlib.sha256()
        for a in (p.q, p.k_pool, p.v_pool, p.block_table, p.seq_lens):
            h.update(a.tobytes())
        assert h.hexdigest() == gold[kvd]["inputs_sha256"]
        out, lse = oracle.decode(p)
        want = np.array([[float.fromhex(x) for x in row] for row in gold[kvd]["lse"]])
        np.testing.assert_allclose(lse, want, rtol=0, atol=1e-14)
        w8 = np.array([float.fromhex(x) for x in gold[kvd]["out_b3_h0_first8"]])
        np.testing.assert_allclose(out[3, 0, :8], w8, rtol=0, atol=1e-15)
