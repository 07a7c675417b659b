"""Helpers for the GPU tests: upload a workload.Problem, run the HIP library through its C ABI, compare."""
import numpy as np
import torch

import paper_2507_01663_amd as ra

ABS_TOL = 1e-2      # max |out_gpu - out_ref| over all elements
REL_TOL = 1e-2      # per (b, h) row: ||out_gpu - out_ref||_2 / ||out_ref||_2
LSE_TOL = 1e-3      # |lse_gpu - lse_ref|


def bits_to_bf16(a, dev):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(dev).view(torch.bfloat16)


class DeviceProblem:
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
        torch.cuda.synchronize()
        return self.out.float().cpu().numpy().astype(np.float64), self.lse.cpu().numpy().astype(np.float64)


def compare(out, lse, ref_out, ref_lse, what="", abs_rel=0.0):
    """Asserts the three tolerances; returns the measured errors.  abs_rel widens the element-wise bound to
    ABS_TOL + abs_rel * |ref| for outputs that are not small: rounding the exact result to bf16 alone moves an
    element by up to 2**-9 of its magnitude, which passes ABS_TOL once |ref| > 5 (prompt prefill: the first tokens of a
    prompt average over few values; a decode step averages over hundreds and never gets there)."""
    assert np.isfinite(out).all(), what + ": non-finite output"
    empty = np.isneginf(ref_lse)
    assert (np.isneginf(lse) == empty).all(), what + ": -inf pattern of lse differs"
    d = out - ref_out
    abs_err = float(np.abs(d).max()) if d.size else 0.0
    num = np.sqrt((d * d).sum(axis=-1))
    den = np.sqrt((ref_out * ref_out).sum(axis=-1))
    rel = np.where(den > 0, num / np.maximum(den, 1e-300), num)
    rel_err = float(rel.max()) if rel.size else 0.0
    lse_err = float(np.abs(lse[~empty] - ref_lse[~empty]).max()) if (~empty).any() else 0.0
    excess = float((np.abs(d) - abs_rel * np.abs(ref_out)).max()) if d.size else 0.0
    assert excess <= ABS_TOL, "%s: max abs err %.3e (%.3e beyond the magnitude allowance)" % (what, abs_err, excess)
    assert rel_err <= REL_TOL, "%s: max row rel err %.3e" % (what, rel_err)
    assert lse_err <= LSE_TOL, "%s: max lse err %.3e" % (what, lse_err)
    return abs_err, rel_err, lse_err
