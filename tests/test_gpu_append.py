"""KV append on the GPU against the oracle, through the C ABI: bit-exact pools and scales over many decode
iterations, then attention over the appended cache."""
import copy

import numpy as np
import pytest
import torch

import oracle
import paper_2507_01663_amd as ra
import workload
from workload.gen import build_problem, f32_to_bf16_bits
from gpu_util import DeviceProblem, compare, bits_to_bf16

pytestmark = pytest.mark.gpu


def growing_problem(kvd, Hq, Hkv, D, lens, steps, seed):
    """A batch whose table rows have pages for `steps` more tokens (fresh pages hold poison, as unused pages do)."""
    lens = np.asarray(lens, dtype=np.int64)
    p = build_problem("append", Hq, Hkv, D, np.zeros(len(lens), dtype=np.int64), 1, lens, kv_dtype=kvd, seed=seed, slack=4.0)
    p = copy.copy(p)
    cols = int((lens.max() + steps + 15) // 16)
    bt = np.full((p.B, cols), -1, dtype=np.int32)
    bt[:, :p.block_table.shape[1]] = p.block_table
    free = iter(sorted(set(range(p.num_pages)) - set(bt[bt >= 0].tolist())))
    for b in range(p.B):
        for i in range(int((lens[b] + 15) // 16), int((lens[b] + steps + 15) // 16)):
            bt[b, i] = next(free)
    p.block_table = bt
    p.k_pool, p.v_pool = np.array(p.k_pool, copy=True), np.array(p.v_pool, copy=True)
    if kvd == "fp8_e4m3":
        p.k_scale, p.v_scale = np.array(p.k_scale, copy=True), np.array(p.v_scale, copy=True)
    p.seq_lens = np.array(p.seq_lens, copy=True)
    return p


def pools_of(dp):
    torch.cuda.synchronize()
    if dp.p.kv_dtype == "bf16":
        k = dp.k_pool.view(torch.int16).cpu().numpy().view(np.uint16)
        v = dp.v_pool.view(torch.int16).cpu().numpy().view(np.uint16)
        return k, v, None, None
    return dp.k_pool.cpu().numpy(), dp.v_pool.cpu().numpy(), dp.k_scale.cpu().numpy(), dp.v_scale.cpu().numpy()


@pytest.mark.parametrize("kvd,Hq,Hkv,D", [("bf16", 28, 4, 128), ("fp8_e4m3", 28, 4, 128), ("fp8_e4m3", 8, 2, 64), ("bf16", 4, 2, 64)])
def test_append_stream_is_bit_exact_and_attention_follows(kvd, Hq, Hkv, D):
    steps = 37  # crosses two page boundaries for every sequence
    lens = [0, 1, 15, 16, 17, 31, 100, 250]
    p = growing_problem(kvd, Hq, Hkv, D, lens, steps, seed=21)
    dec = ra.Decoder(0)
    dp = DeviceProblem(p)
    r = np.random.default_rng(77)
    for t in range(steps):
        # magnitudes wander, so that some rows keep the page's scale and some force a re-quantisation
        amp = (0.2 * np.exp(r.normal(0.0, 0.6, size=(p.B, Hkv, 1)))).astype(np.float32)  # stays near the N(0,1) range the tolerances assume
        kn = f32_to_bf16_bits((r.standard_normal((p.B, Hkv, D)).astype(np.float32) * amp))
        vn = f32_to_bf16_bits((r.standard_normal((p.B, Hkv, D)).astype(np.float32) * amp))
        assert oracle.append(p, kn, vn) == 0
        dec.append(dp.c, bits_to_bf16(kn, "cuda:0"), bits_to_bf16(vn, "cuda:0"))
        p.seq_lens += 1
        dp.seq_lens += 1
        if t in (0, 15, 16, steps - 1):
            k, v, ks, vs = pools_of(dp)
            np.testing.assert_array_equal(k, p.k_pool, err_msg="K pool after step %d" % t)
            np.testing.assert_array_equal(v, p.v_pool, err_msg="V pool after step %d" % t)
            if ks is not None:
                np.testing.assert_array_equal(ks, p.k_scale, err_msg="K scales after step %d" % t)
                np.testing.assert_array_equal(vs, p.v_scale, err_msg="V scales after step %d" % t)
    # the cache the library wrote serves the library's attention, checked against the oracle on the oracle's cache
    dec.decode(dp.c)
    ref_out, ref_lse = oracle.decode(p)
    compare(*dp.results(), ref_out, ref_lse, "attention after %d appends (%s)" % (steps, kvd))


def test_append_skips_what_it_must_not_write():
    p = growing_problem("bf16", 4, 2, 64, [5, 20, 33], 1, seed=3)
    p.seq_lens[0] = p.block_table.shape[1] * 16      # no room in the table row
    p.seq_lens[1] = -3
    p.block_table[2, 33 // 16] = p.num_pages          # page id out of range
    dp = DeviceProblem(p)
    k0, v0, _, _ = pools_of(dp)
    dec = ra.Decoder(0)
    z = torch.ones(p.B, p.Hkv, p.D, dtype=torch.bfloat16, device="cuda:0")
    dec.append(dp.c, z, z)
    k1, v1, _, _ = pools_of(dp)
    np.testing.assert_array_equal(k1, k0)
    np.testing.assert_array_equal(v1, v0)
    with pytest.raises(ra.RolloutAttnError):
        ra.rollout_attn_append(dec.ctx, dp.c, None, None, None)
