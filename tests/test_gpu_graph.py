"""The decode step, the KV append and the prompt prefill only enqueue kernels on the caller's stream (no allocation, no
memset, no synchronisation), so a caller may record them into a HIP graph.  Every replay is checked: against the
oracle where inputs change between replays, bit for bit against the eager call otherwise, with eager work and
synchronisations of the program's own between the replays."""
import numpy as np
import pytest
import torch

import oracle
import workload
from gpu_util import DeviceProblem, bits_to_bf16, compare

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dec():
    import paper_2507_01663_amd as ra
    d = ra.Decoder(0)
    yield d
    d.close()


def capture(fn):
    """Records what fn enqueues on a side stream into a graph."""
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=s):
        fn()
    return g


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8_e4m3"])
def test_decode_step_replayed_from_a_graph(dec, kv_dtype):
    p = workload.make_problem("mid7b", seed=3, kv_dtype=kv_dtype)
    dp = DeviceProblem(p)
    dec.decode(dp.c)                       # the decoder's workspace exists before the capture
    torch.cuda.synchronize()
    g = capture(lambda: dec.decode(dp.c))
    for rep in range(4):
        # other queries, and some sequences a token shorter, each time: the graph reads them from the same buffers
        p.q = workload.normal_bf16(p.q.size, 200 + rep, 1).reshape(p.q.shape)
        shrink = (np.arange(p.B) % 3 == rep % 3) & (p.seq_lens % 16 >= 2)   # stays in its last page and above the prompt
        p.seq_lens = (p.seq_lens - shrink).astype(np.int32)
        dp.q.copy_(bits_to_bf16(p.q, "cuda:0"))
        dp.seq_lens.copy_(torch.from_numpy(p.seq_lens))
        dp.out.fill_(float("nan"))
        dp.lse.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        got = dp.results()
        compare(*got, *oracle.decode(p), "%s replay %d" % (kv_dtype, rep))
        # the eager call on the same inputs gives the same bytes
        dp.out.fill_(float("nan"))
        dec.decode(dp.c)
        eager = dp.results()
        assert (eager[0] == got[0]).all() and (eager[1] == got[1]).all(), "replay %d differs from the eager call" % rep


def test_append_and_prefill_replayed_from_a_graph(dec):
    from test_gpu_prefill import DevicePrefill
    b = workload.make_prefill("mid7b", seed=1)
    d = DevicePrefill(b, kv_dtype="bf16")
    dec.prefill(d.c)
    torch.cuda.synchronize()
    ref = [t.clone() for t in (d.out, d.lse, d.k_pool, d.v_pool)]
    g = capture(lambda: dec.prefill(d.c))
    for rep in range(3):
        for t in (d.out, d.lse, d.k_pool, d.v_pool):   # as they were before the eager call
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for name, t, r in zip(("out", "lse", "k_pool", "v_pool"), (d.out, d.lse, d.k_pool, d.v_pool), ref):
            same = (t.view(torch.int16) == r.view(torch.int16)) if t.dtype == torch.bfloat16 else (t == r)
            assert bool(same.all()), "prefill replay %d: %s differs from the eager call" % (rep, name)

    # append: the new token's K and V rows land where the eager call puts them
    p = workload.make_problem("mid7b", seed=4)
    p.seq_lens = np.where(p.seq_lens % 16 == 0, p.seq_lens - 1, p.seq_lens).astype(np.int32)  # room in the last page
    dp = DeviceProblem(p)
    Hkv = p.Hkv
    k_new = bits_to_bf16(workload.normal_bf16(p.B * Hkv * p.D, 301, 1).reshape(p.B, Hkv, p.D), "cuda:0")
    v_new = bits_to_bf16(workload.normal_bf16(p.B * Hkv * p.D, 302, 1).reshape(p.B, Hkv, p.D), "cuda:0")
    k0, v0 = dp.k_pool.clone(), dp.v_pool.clone()
    dec.append(dp.c, k_new, v_new)
    torch.cuda.synchronize()
    k1, v1 = dp.k_pool.clone(), dp.v_pool.clone()
    assert not bool((k1.view(torch.int16) == k0.view(torch.int16)).all())
    g = capture(lambda: dec.append(dp.c, k_new, v_new))
    for rep in range(3):
        dp.k_pool.copy_(k0)
        dp.v_pool.copy_(v0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert bool((dp.k_pool.view(torch.int16) == k1.view(torch.int16)).all()), "append replay %d: K differs" % rep
        assert bool((dp.v_pool.view(torch.int16) == v1.view(torch.int16)).all()), "append replay %d: V differs" % rep
