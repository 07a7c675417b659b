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
