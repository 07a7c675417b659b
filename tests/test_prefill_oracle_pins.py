"""Pins for the prefill oracle (CPU only): causal attention of packed prompts, against torch's fp64 scaled dot
product attention with a causal mask, against the decode oracle (the last token of a prompt is a decode step
over the prompt's cache), and closed forms."""
import numpy as np
import torch

import oracle
import workload
from workload.gen import bf16_bits_to_f32, f32_to_bf16_bits, build_problem


def rand_bits(shape, seed, scale=1.0):
    return f32_to_bf16_bits((np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32))


def test_matches_library_causal_sdpa_in_fp64():
    Hq, Hkv, D = 6, 2, 32
    cu = np.array([0, 1, 18, 50], dtype=np.int32)
    q, k, v = rand_bits((50, Hq, D), 1), rand_bits((50, Hkv, D), 2), rand_bits((50, Hkv, D), 3)
    scale = 0.17
    out, lse = oracle.prefill(q, k, v, cu, scale)
    for g in range(3):
        a, b = cu[g], cu[g + 1]
        Q = torch.from_numpy(bf16_bits_to_f32(q[a:b]).astype(np.float64)).permute(1, 0, 2)                       # [Hq, n, D]
        K = torch.from_numpy(bf16_bits_to_f32(k[a:b]).astype(np.float64)).permute(1, 0, 2).repeat_interleave(Hq // Hkv, 0)
        V = torch.from_numpy(bf16_bits_to_f32(v[a:b]).astype(np.float64)).permute(1, 0, 2).repeat_interleave(Hq // Hkv, 0)
        ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V, is_causal=True, scale=float(np.float32(scale)))
        np.testing.assert_allclose(out[a:b], ref.permute(1, 0, 2).numpy(), rtol=1e-12, atol=1e-13)
        S = (Q @ K.transpose(1, 2)) * float(np.float32(scale))
        S = S.masked_fill(~torch.tril(torch.ones(b - a, b - a, dtype=torch.bool)), float("-inf"))
        np.testing.assert_allclose(lse[a:b], torch.logsumexp(S, -1).T.numpy(), rtol=1e-12, atol=1e-13)


def test_first_token_sees_only_itself_and_future_tokens_do_not_matter():
    Hq, Hkv, D = 4, 2, 16
    cu = np.array([0, 9], dtype=np.int32)
    q, k, v = rand_bits((9, Hq, D), 4), rand_bits((9, Hkv, D), 5), rand_bits((9, Hkv, D), 6)
    out, lse = oracle.prefill(q, k, v, cu, 0.25)
    # token 0: one key, so out = v_0 and lse = its score
    for h in range(Hq):
        np.testing.assert_array_equal(out[0, h], bf16_bits_to_f32(v[0, h // 2]).astype(np.float64))
        s = 0.25 * float(np.dot(bf16_bits_to_f32(q[0, h]).astype(np.float64), bf16_bits_to_f32(k[0, h // 2]).astype(np.float64)))
        assert abs(lse[0, h] - s) < 1e-12
    # changing the keys and values after position 4 leaves tokens 0..4 alone
    k2, v2 = k.copy(), v.copy()
    k2[5:], v2[5:] = rand_bits((4, Hkv, D), 7), rand_bits((4, Hkv, D), 8)
    out2, lse2 = oracle.prefill(q, k2, v2, cu, 0.25)
    np.testing.assert_array_equal(out2[:5], out[:5])
    np.testing.assert_array_equal(lse2[:5], lse[:5])
    assert np.abs(out2[5:] - out[5:]).max() > 1e-3


def test_last_prompt_token_is_a_decode_step_over_the_prompts_cache():
    # a batch of sequences with no response: decode attention of the last prompt token over the paged prompt
    p = build_problem("pf", 8, 2, 64, [48, 32], 1, [0, 0], seed=11)
    T = int(p.seq_lens.sum())
    cu = np.concatenate([[0], np.cumsum(p.seq_lens)]).astype(np.int32)
    k = np.empty((T, p.Hkv, p.D), dtype=np.uint16)
    v = np.empty_like(k)
    for b in range(p.B):
        for kv in range(p.Hkv):
            kk, vv, _ = oracle.gather(p, b, kv)
            k[cu[b]:cu[b + 1], kv], v[cu[b]:cu[b + 1], kv] = kk, vv
    q = rand_bits((T, p.Hq, p.D), 12)
    q[cu[1:] - 1] = p.q                                    # the decode queries sit at the last positions
    out, lse = oracle.prefill(q, k, v, cu, p.softmax_scale)
    dout, dlse = oracle.decode(p)
    np.testing.assert_allclose(out[cu[1:] - 1], dout, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse[cu[1:] - 1], dlse, rtol=1e-12, atol=1e-14)


# ---- the cache write (oracle.prefill_write) --------------------------------------------------------------------

def _fresh_pools(b, fp8):
    shape = (b.num_pages, b.Hkv, 16, b.D)
    if fp8:
        return (np.full(shape, 0x7F, np.uint8), np.full(shape, 0x7F, np.uint8),
                np.full(shape[:2], np.nan, np.float32), np.full(shape[:2], np.nan, np.float32))
    return np.full(shape, 0x7FC0, np.uint16), np.full(shape, 0x7FC0, np.uint16), None, None


def test_cache_write_bf16_is_a_scatter_of_the_rows():
    b = workload.build_prefill("pw", 4, 2, 32, [1, 16, 17, 0, 50], seed=3)
    kp, vp, _, _ = _fresh_pools(b, False)
    oracle.prefill_write(b.k, b.v, b.cu_seqlens, b.page_offsets, b.pages, kp, vp)
    # brute force, token by token, in numpy indexing
    ek, ev, _, _ = _fresh_pools(b, False)
    for g in range(b.lens.size):
        for i in range(int(b.lens[g])):
            pid = b.pages[b.page_offsets[g] + i // 16]
            ek[pid, :, i % 16] = b.k[b.cu_seqlens[g] + i]
            ev[pid, :, i % 16] = b.v[b.cu_seqlens[g] + i]
    np.testing.assert_array_equal(kp, ek)
    np.testing.assert_array_equal(vp, ev)
    # pages nobody lists and the empty slots of last pages keep their poison
    assert (kp == 0x7FC0).sum() == kp.size - int(b.lens.sum()) * b.Hkv * b.D


def test_cache_write_e4m3_full_pages_equal_the_input_generators_tiles():
    from workload.gen import _quantise_tiles
    b = workload.build_prefill("pw", 4, 2, 64, [64, 32], seed=5)          # whole pages only
    kp, vp, ks, vs = _fresh_pools(b, True)
    oracle.prefill_write(b.k, b.v, b.cu_seqlens, b.page_offsets, b.pages, kp, vp, ks, vs)
    for src, pool, sc in ((b.k, kp, ks), (b.v, vp, vs)):
        for g in range(2):
            for pi in range(int(b.lens[g]) // 16):
                pid = b.pages[b.page_offsets[g] + pi]
                rows = src[b.cu_seqlens[g] + 16 * pi:b.cu_seqlens[g] + 16 * pi + 16]      # [16, Hkv, D]
                tiles = rows.transpose(1, 0, 2).reshape(b.Hkv, 16 * b.D)
                codes, scale = _quantise_tiles(tiles)                                        # the generator's whole-page rule
                np.testing.assert_array_equal(pool[pid].reshape(b.Hkv, -1), codes)
                np.testing.assert_array_equal(sc[pid].view(np.uint32), scale.view(np.uint32))


def test_cache_write_e4m3_error_bound_partial_pages_and_zero_rows():
    b = workload.build_prefill("pw", 2, 2, 32, [21, 16, 5], seed=8)
    k = bf16_bits_to_f32(b.k).copy()
    k[21:37] = 0.0                        # prompt 1 is one page of zero keys: scale 1, codes 0
    k[3] *= 300.0                         # one large row sets page 0's scale
    b.k = f32_to_bf16_bits(k)
    kp, vp, ks, vs = _fresh_pools(b, True)
    oracle.prefill_write(b.k, b.v, b.cu_seqlens, b.page_offsets, b.pages, kp, vp, ks, vs)
    tab = oracle.e4m3_decode_table()
    for src, pool, sc in ((b.k, kp, ks), (b.v, vp, vs)):
        x = bf16_bits_to_f32(src).astype(np.float64)
        for g in range(3):
            n = int(b.lens[g])
            for pi in range((n + 15) // 16):
                pid = b.pages[b.page_offsets[g] + pi]
                rows = x[b.cu_seqlens[g] + 16 * pi:b.cu_seqlens[g] + min(n, 16 * pi + 16)]      # [r, Hkv, D]
                r = rows.shape[0]
                for kv in range(b.Hkv):
                    amax = np.abs(rows[:, kv]).max()
                    s = float(sc[pid, kv])
                    # scale = absmax over the rows written (not over the poison in the unfilled slots) / 448, in binary32
                    assert s == (float(np.float32(amax) / np.float32(448.0)) if amax > 0 else 1.0)
                    deq = tab[pool[pid, kv, :r]] * s
                    # half a step of the format at that magnitude (3 mantissa bits: step <= |y|/8; 2^-9 below 2^-6)
                    y = np.abs(rows[:, kv]) / s
                    step = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(y, 2.0 ** -6))) - 3), 2.0 ** -9)
                    assert (np.abs(deq - rows[:, kv]) <= (0.5 * step + 1e-6 * y) * s + 1e-12).all()
                    assert (pool[pid, kv, r:] == 0x7F).all()        # unfilled slots untouched
                    if amax > 0:
                        assert np.abs(tab[pool[pid, kv, :r]]).max() == 448.0      # the largest element maps to the top code
    # the zero page
    pid = b.pages[b.page_offsets[1]]
    assert (kp[pid] == 0).all() and (ks[pid] == 1.0).all()
    # a page no prompt lists keeps its poison and its scale
    unused = sorted(set(range(b.num_pages)) - set(int(x) for x in b.pages))
    assert unused and (kp[unused] == 0x7F).all() and np.isnan(ks[unused]).all()


def test_cache_write_skips_bad_page_ids_and_tokens_beyond_the_list():
    b = workload.build_prefill("pw", 2, 1, 16, [40], seed=2)
    pages = b.pages[:2].copy()            # room for 32 of the 40 tokens
    pages[1] = b.num_pages + 3            # and the second id is out of range
    kp, vp, _, _ = _fresh_pools(b, False)
    oracle.prefill_write(b.k, b.v, b.cu_seqlens, np.array([0, 2], np.int32), pages, kp, vp)
    assert (kp != 0x7FC0).sum() <= 16 * b.D and np.array_equal(kp[pages[0], 0], b.k[:16, 0])
    assert np.array_equal(vp[pages[0], 0], b.v[:16, 0])
