"""Device-memory plumbing over torch for callers of the binding: uploads a host-side batch description (any object
with the fields of ``workload.Problem``) and fills the ``ra_problem`` that the C ABI takes.  No arithmetic here."""
import numpy as np
import torch

from . import binding as ra


def bits_to_bf16(a, dev):
    """uint16 bit patterns (numpy) -> a bf16 tensor on dev."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(dev).view(torch.bfloat16)


class DeviceProblem:
    """The tensors of one decode step on the device and its ``ra_problem`` (``.c``)."""

    def __init__(self, p, dev="cuda:0", flags=0, use_hint=True, share_pools_with=None):
        self.p = p
        self.q = bits_to_bf16(p.q, dev)
        if share_pools_with is not None:
            o = share_pools_with
            self.k_pool, self.v_pool, self.k_scale, self.v_scale = o.k_pool, o.v_pool, o.k_scale, o.v_scale
        elif p.kv_dtype == "bf16":
            self.k_pool, self.v_pool = bits_to_bf16(p.k_pool, dev), bits_to_bf16(p.v_pool, dev)
            self.k_scale = self.v_scale = None
        else:
            self.k_pool, self.v_pool = torch.from_numpy(p.k_pool).to(dev), torch.from_numpy(p.v_pool).to(dev)
            self.k_scale, self.v_scale = torch.from_numpy(p.k_scale).to(dev), torch.from_numpy(p.v_scale).to(dev)
        self.block_table = torch.from_numpy(p.block_table).to(dev)
        self.seq_lens = torch.from_numpy(p.seq_lens).to(dev)
        self.seq_group = torch.from_numpy(p.seq_group).to(dev)
        self.pfx_off = torch.from_numpy(p.prefix_page_offsets).to(dev)
        self.pfx_pages = torch.from_numpy(p.prefix_pages).to(dev) if p.prefix_pages.size else torch.zeros(1, dtype=torch.int32, device=dev)
        self.out = torch.full((p.B, p.Hq, p.D), float("nan"), dtype=torch.bfloat16, device=dev)
        self.lse = torch.full((p.B, p.Hq), float("nan"), dtype=torch.float32, device=dev)
        self.set(flags, use_hint)

    def set(self, flags=0, use_hint=True):
        hint = dict(seq_group=self.seq_group, prefix_page_offsets=self.pfx_off, prefix_pages=self.pfx_pages) if use_hint else {}
        self.c = ra.problem_from_tensors(self.q, self.k_pool, self.v_pool, self.block_table, self.seq_lens, self.out, self.lse,
                                         float(self.p.softmax_scale), k_scale=self.k_scale, v_scale=self.v_scale, flags=flags, **hint)
        return self

    def results(self):
        """(out, lse) as float64 numpy arrays, after the device has finished."""
        torch.cuda.synchronize()
        return self.out.float().cpu().numpy().astype(np.float64), self.lse.cpu().numpy().astype(np.float64)
