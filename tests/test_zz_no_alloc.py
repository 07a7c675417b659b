"""rollout_attn_decode_static (the decode step on the library's built-in workspace, for callers that cannot
allocate) against rollout_attn_decode on the same inputs, through the C ABI: two calls in a row, the second on a
smaller problem, the results byte for byte those of the workspace entry point and within tolerance of the oracle;
a shape whose workspace exceeds the built-in one is refused."""
import numpy as np
import pytest
import torch

import oracle
import paper_2507_01663_amd as ra
import workload
from gpu_util import DeviceProblem, compare

pytestmark = pytest.mark.gpu


def test_static_workspace_entry_point_matches_the_workspace_one():
    dec = ra.Decoder(0)
    try:
        for name, kv in (("mid7b", "bf16"), ("tiny", "bf16"), ("mid32b", "fp8_e4m3"), ("tiny", "fp8_e4m3")):
            p = workload.make_problem(name, seed=3, kv_dtype=kv)
            print("case", name, kv, "B", p.B, flush=True)
            ref = DeviceProblem(p)
            dec.decode(ref.c)                       # caller-provided workspace
            got = DeviceProblem(p)
            before = torch.cuda.memory_allocated(0)
            dec.decode_static(got.c)                # built-in workspace
            torch.cuda.synchronize()
            assert torch.cuda.memory_allocated(0) == before
            assert torch.equal(ref.out.view(torch.int16), got.out.view(torch.int16)), (name, kv)
            assert torch.equal(ref.lse, got.lse), (name, kv)
            compare(*got.results(), *oracle.decode(p), "%s %s on the built-in workspace" % (name, kv))
        # a batch whose partial results do not fit the built-in workspace is refused, and nothing runs
        small = DeviceProblem(workload.make_problem("tiny", seed=0))
        small.c.B = 1 << 16
        with pytest.raises(ra.RolloutAttnError) as e:
            dec.decode_static(small.c)
        assert e.value.status == ra.RA_ERR_WORKSPACE_TOO_SMALL and "built-in" in str(e.value)
        torch.cuda.synchronize()
        assert torch.isnan(small.out.float()).all()
    finally:
        dec.close()
