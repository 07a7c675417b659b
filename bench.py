#!/usr/bin/env python3
"""Benchmark of the rollout_attn decode step on one MI355X.

A step is one rollout_attn_decode call over the whole batch (schedule + attention + merge = one layer's
attention for one generated token).  The workload is the 7B-shaped GRPO batch (32 prompts x 8 responses,
Hq=28, Hkv=4, D=128, prompt 512, responses U[0,3584], page 16, pages randomly permuted).  Several
independent instances (own pools and tables, distinct seeds) are resident in HBM and the timed loop rotates
over them, so no step finds its pages in the 256 MB last-level cache.

Prints ONE JSON line: whole-step throughput in algorithmic GB/s (every distinct KV token once, shared
prompt pages once per group), steps/s, the roofline of the dominant kernel from HIP events, what a pure
streaming probe of the same access pattern reaches on this device (the practical ceiling), and the fp64
oracle timed on the host cores as a reported baseline.  The default run also carries, from child processes
that run before this one touches the GPU: the same workload with an e4m3 cache, the 32B-shaped long-tail
batch, and the 72B-shaped streaming batch over its 64 consecutive steps.
"""
import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published


def kernel_source_hash():
    import hashlib
    h = hashlib.sha256()
    for f in ("ra_kernels.hip", "ra_device.h", "ra_internal.h"):
        h.update(open(os.path.join(ROOT, "paper_2507_01663_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:16]


def recorded_traffic(workload_name):
    """HBM bytes per launch of the attention kernel from the committed rocprofv3 --pmc runs, if they were taken
    on the current kernel source; else None."""
    path = os.path.join(ROOT, "profiles", "attention_traffic.json")
    try:
        rec = json.load(open(path))
    except (OSError, ValueError):
        return None
    ent = rec.get(workload_name)   # keyed by workload and variant, e.g. "grpo7b", "grpo7b_fp8"
    if not ent or ent.get("kernel_source_hash") != kernel_source_hash():
        return None
    return ent.get("hbm_bytes_per_launch")


def child_summary(extra, timeout=600):
    """Runs this script in a process of its own and returns the fields of its line that the parent reports."""
    cmd = [sys.executable, os.path.abspath(__file__), "--no-cpu-baseline", "--child"] + extra
    try:
        r = subprocess.run(cmd, capture_output=True, text=True, timeout=timeout)
        e = json.loads([l for l in r.stdout.splitlines() if l.startswith("{")][-1])
        keep = ("value", "unit", "ms_per_step", "steps_per_s", "pct_of_hbm_peak", "phases_ms", "roofline", "schedule_reused", "two_streams", "consecutive_steps")
        out = {k: e[k] for k in keep if k in e}
        out["workload"] = e["config"]["workload"]
        out["algorithmic_MB_per_step"] = e["config"]["algorithmic_MB_per_step"]
        return out
    except Exception as exc:  # the parent's own line is the contract; say what happened to the extra run
        return {"error": "%s: %s" % (type(exc).__name__, exc)}


def row_errors(out, lse, ref_out, ref_lse):
    """(max abs, max row-relative, max lse) error of a result against the oracle's."""
    import numpy as np
    d = out - ref_out
    num = np.sqrt((d * d).sum(axis=-1))
    den = np.sqrt((ref_out * ref_out).sum(axis=-1))
    rel = np.where(den > 0, num / np.maximum(den, 1e-300), num)
    fin = np.isfinite(ref_lse)
    return float(np.abs(d).max()), float(rel.max()), float(np.abs(lse[fin] - ref_lse[fin]).max()) if fin.any() else 0.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="grpo7b")
    ap.add_argument("--kv-dtype", default="bf16")
    ap.add_argument("--instances", type=int, default=4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sharing", action="store_true", help="ignore the prompt-group hint (A/B)")
    ap.add_argument("--calibrate-copy", action="store_true", help="also run three 1 GiB device copies (counter calibration)")
    ap.add_argument("--no-extras", "--no-e4m3", dest="no_extras", action="store_true",
                    help="leave out the child-process runs (e4m3 cache, tail32b, stream72b) and the two-stream run that the default "
                         "run appends (a profiler then sees the one-stream steps alone, no launches that overlap)")
    ap.add_argument("--consecutive", action="store_true",
                    help="streaming workloads: time the configuration's consecutive decode steps one after the other, each with "
                         "its own lengths, block table and queries uploaded before it (the upload timed separately)")
    ap.add_argument("--weight-copy", action="store_true",
                    help="stream host-to-device copies on a second stream during the timed steps (the device-visible side "
                         "of an asynchronous weight update) and report both rates")
    ap.add_argument("--child", action="store_true", help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: one GPU only. Sequences are independent, so the path shards over GPUs with no exchange "
              "and one GPU's throughput on its share is the figure; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    # The other configurations are measured first, each by a child process of its own (started before this process
    # touches the GPU), and reported beside the headline figures, never mixed into `value`.
    extras = {}
    plain = (args.kv_dtype == "bf16" and args.workload == "grpo7b" and not args.no_extras and not args.no_sharing and not args.weight_copy
             and not args.calibrate_copy and not args.child and not args.consecutive)
    if plain:
        extras["e4m3_kv"] = child_summary(["--workload", args.workload, "--kv-dtype", "fp8_e4m3", "--steps", str(args.steps),
                                           "--warmup", str(args.warmup), "--instances", str(args.instances)])
        extras["e4m3_kv"]["note"] = "K/V stored as e4m3 codes with per-page-per-head fp32 scales, same lengths and tables"
        extras["tail32b"] = child_summary(["--workload", "tail32b", "--steps", "80", "--warmup", "10"])
        extras["stream72b"] = child_summary(["--workload", "stream72b", "--consecutive"])

    import numpy as np
    import torch
    import paper_2507_01663_amd as ra
    import workload
    from paper_2507_01663_amd.torch_util import DeviceProblem, bits_to_bf16

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    ra.load_library()                                  # fails loudly when the HIP library is not built
    dec = ra.Decoder(0)
    flags = ra.RA_FLAG_NO_PREFIX_SHARING if args.no_sharing else 0
    stream = torch.cuda.current_stream(0)
    cfg = workload.CONFIGS[args.workload]
    name = args.workload + ("" if args.kv_dtype == "bf16" else "_fp8")

    if args.consecutive:
        consecutive_steps(args, cfg, name, dec, stream, flags)
        return

    t0 = time.time()
    probs, devs = [], []
    if cfg["resp"] == "stream":
        # streaming workload: one static pool; the instances are decode steps spread over the run, each with its
        # own lengths, block table (re-drawn from the seed) and queries
        steps = sorted(set(int(round(i * (cfg["steps"] - 1) / max(1, args.instances - 1))) for i in range(args.instances)))
        width = (cfg["prompt"] + cfg["resp_max"] + cfg["steps"]) // 16 + 1
        for i, st in enumerate(steps):
            p = workload.make_problem(args.workload, seed=0, step=st, kv_dtype=args.kv_dtype, make_values=(i == 0),
                                      pool=None if i == 0 else (probs[0].k_pool, probs[0].v_pool, probs[0].k_scale, probs[0].v_scale),
                                      num_pages=None if i == 0 else probs[0].num_pages)
            bt = np.full((p.B, width), -1, dtype=np.int32)
            bt[:, :p.block_table.shape[1]] = p.block_table
            p.block_table, p.max_pages_per_seq = bt, width
            if p.q is None:
                p.q = workload.normal_bf16(p.B * p.Hq * p.D, 0, 1000 + st).reshape(p.B, p.Hq, p.D)
            probs.append(p)
            devs.append(DeviceProblem(p, flags=flags, share_pools_with=devs[0] if i else None))
    else:
        for i in range(args.instances):
            p = workload.make_problem(args.workload, seed=i, kv_dtype=args.kv_dtype)
            probs.append(p)
            devs.append(DeviceProblem(p, flags=flags))
    if args.calibrate_copy:
        # a plain copy of known size in the same process, so that a counter run can scale its byte counters
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    alg_bytes = [p.algorithmic_bytes(share_prefix=True) for p in probs]
    print("# %d instances of %s generated and uploaded in %.1f s; algorithmic MB/step: %s" %
          (args.instances, args.workload, time.time() - t0, [round(b / 1e6, 1) for b in alg_bytes]), file=sys.stderr)

    def run(n, first=0):
        for i in range(n):
            dec.decode(devs[(first + i) % len(devs)].c, stream)

    run(args.warmup)
    torch.cuda.synchronize()
    copy_info = None
    if args.weight_copy:
        # enough 256 MiB host-to-device copies, queued on a stream of their own (default priority), to outlast the steps
        chunk = 1 << 28
        host = torch.empty(chunk, dtype=torch.uint8, pin_memory=True)
        dev_w = torch.empty(chunk, dtype=torch.uint8, device="cuda:0")
        side = torch.cuda.Stream(device=0)
        t_est = args.steps * 0.3e-3 if cfg["resp"] != "stream" and args.workload != "tail32b" else args.steps * 2.5e-3
        ncopies = max(4, int(t_est * 60e9 / chunk) + 4)
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(side):
            c0.record(side)
            for _ in range(ncopies):
                dev_w.copy_(host, non_blocking=True)
            c1.record(side)
    t0 = time.perf_counter()
    run(args.steps)
    stream.synchronize()
    wall = time.perf_counter() - t0
    if args.weight_copy:
        torch.cuda.synchronize()
        copy_s = c0.elapsed_time(c1) * 1e-3
        copy_info = {"host_to_device_GBps": round(ncopies * chunk / copy_s / 1e9, 1), "copies": ncopies, "copy_seconds": round(copy_s, 4),
                     "steps_seconds": round(wall, 4), "note": "the copies ran for the whole of the timed steps" if copy_s >= wall else
                     "the copies ended before the timed steps did"}
    torch.cuda.synchronize()
    total_bytes = sum(alg_bytes[i % len(devs)] for i in range(args.steps))
    ms_per_step = wall * 1e3 / args.steps
    gbps = total_bytes / wall / 1e9

    # per-kernel durations from HIP events recorded by the library on the same stream, over the same steps
    ra.rollout_attn_set_timing(dec.ctx, True)
    run(min(args.warmup, 8))
    phase = np.zeros(3)
    att_bytes = 0
    for i in range(args.steps):
        dec.decode(devs[i % len(devs)].c, stream)
        phase += np.array(ra.rollout_attn_get_timing(dec.ctx))
        att_bytes += alg_bytes[i % len(devs)]
    ra.rollout_attn_set_timing(dec.ctx, False)
    phase /= args.steps
    att_gbps = att_bytes / args.steps / (phase[1] * 1e-3) / 1e9

    out = {
        "metric": "decode_attn_hbm_GBps", "value": round(gbps, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if args.kv_dtype == "bf16" else "fp8_e4m3 KV, bf16 MFMA", "data": "synthetic",
        "steps_per_s": round(args.steps / wall, 1), "pct_of_hbm_peak": round(100 * gbps / HBM_PEAK_GBPS, 2),
        "config": {"workload": name, "B": probs[0].B, "Hq": probs[0].Hq,
                   "Hkv": probs[0].Hkv, "D": probs[0].D, "page": 16, "instances": args.instances,
                   "prefix_sharing": not args.no_sharing,
                   "algorithmic_MB_per_step": round(sum(alg_bytes) / len(alg_bytes) / 1e6, 2),
                   "kv_tokens_per_step": int(sum(p.kv_tokens() for p in probs) / len(probs))},
        "phases_ms": {"schedule": round(float(phase[0]), 5), "attention": round(float(phase[1]), 5),
                      "merge": round(float(phase[2]), 5),
                      "note": "HIP events around the library's launches (each record adds a few microseconds to the phase it "
                              "ends); batches of up to 512 sequences are scheduled inside the attention kernel: no schedule "
                              "launch, `schedule` is 0 and its time is part of `attention`"},
        "roofline": {"bound": "hbm", "kernel": "attention_kernel", "achieved": round(att_gbps, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(att_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": recorded_traffic(name + ("_noshare" if args.no_sharing else ""))},
    }
    if copy_info:
        out["weight_copy"] = copy_info

    # What the memory system delivers to this access pattern with no arithmetic at all: the attention kernel's grid
    # and LDS ring streaming 4 KB tiles from scattered places (its own pattern), and consecutive ones.  The buffer is
    # as large as the K/V pools the timed steps rotate through (a power of two, 4 to 64 GiB: what the probe reaches
    # falls with the memory it ranges over, 7.1 TB/s over 1 GiB, 6.5-6.65 from 16 GiB up), a launch reads what a step does.
    pools = {}
    for d in devs:
        for t in (d.k_pool, d.v_pool):
            pools[t.data_ptr()] = t.numel() * t.element_size()
    footprint = sum(pools.values())
    buf_log2 = min(36, max(32, (footprint - 1).bit_length()))
    buf = torch.empty(1 << buf_log2, dtype=torch.uint8, device="cuda:0")
    buf.random_(0, 255)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    import ctypes
    sp = ctypes.c_void_p(stream.cuda_stream)
    waves = ra.rollout_attn_wave_count(dec.ctx, ra.RA_KV_BF16, 128)
    entries = max(1, int(round(sum(alg_bytes) / len(alg_bytes) / (waves * 16384))))
    ceil = {}
    for label, scattered in (("gather_4KB_tiles", 1), ("sequential", 0), ("gather_plain_loads", 3), ("sequential_plain_loads", 2)):
        for _ in range(3):
            n = ra.rollout_attn_debug_stream(dec.ctx, ctypes.c_void_p(buf.data_ptr()), buf.numel(), 4096, scattered, entries, sp)
        ev0.record(stream)
        for _ in range(10):
            n = ra.rollout_attn_debug_stream(dec.ctx, ctypes.c_void_p(buf.data_ptr()), buf.numel(), 4096, scattered, entries, sp)
        ev1.record(stream)
        torch.cuda.synchronize()
        ceil[label] = n / (ev0.elapsed_time(ev1) / 10) / 1e6
    # the same scattered stream with its last eighth (and quarter) handed out at run time in chunks of 4 entries
    # (64 KB, the size of eight pages of one kv head): does evening out the waves' end times buy anything?
    tail = {}
    for frac in (8, 4):
        static = entries - entries // frac
        for _ in range(3):
            n = ra.rollout_attn_debug_stream_tail(dec.ctx, ctypes.c_void_p(buf.data_ptr()), buf.numel(), entries, static, 4, sp)
        ev0.record(stream)
        for _ in range(10):
            n = ra.rollout_attn_debug_stream_tail(dec.ctx, ctypes.c_void_p(buf.data_ptr()), buf.numel(), entries, static, 4, sp)
        ev1.record(stream)
        torch.cuda.synchronize()
        tail["last_1/%d_ticketed_GBps" % frac] = round(n / (ev0.elapsed_time(ev1) / 10) / 1e6, 1)
    del buf
    out["stream_ceiling"] = {"GBps": round(ceil["gather_4KB_tiles"], 1), "sequential_GBps": round(ceil["sequential"], 1), "unit": "GB/s",
                             "buffer_GiB": 1 << (buf_log2 - 30), "kv_pools_GiB": round(footprint / 2**30, 2),
                             "MB_per_launch": round(entries * waves * 16384 / 1e6, 1),
                             "pct_of_hbm_peak": round(100 * ceil["gather_4KB_tiles"] / HBM_PEAK_GBPS, 2),
                             "note": "read-only probe with the attention kernel's grid and LDS ring, no arithmetic: 4 KB tiles from "
                                     "scattered places (the kernel's own pattern) and from consecutive ones, by loads with the "
                                     "non-temporal hint as the kernel's page loads are; measured in this run",
                             "without_the_hint": {"GBps": round(ceil["gather_plain_loads"], 1),
                                                  "sequential_GBps": round(ceil["sequential_plain_loads"], 1)},
                             "ticketed_tail": dict(tail, note="the scattered stream again, its end handed out at run time through an "
                                                              "atomic counter in chunks of 64 KB instead of split evenly beforehand")}
    out["pct_of_ceiling"] = round(100 * gbps / ceil["gather_4KB_tiles"], 2)
    out["roofline"]["frac_of_ceiling"] = round(att_gbps / ceil["gather_4KB_tiles"], 4)

    # A model calls the step once per layer with the same lengths and groups; all layers but the first can take the
    # first one's schedule (RA_FLAG_REUSE_SCHEDULE).  Reported beside `value`, which always includes the schedule:
    # every instance gets a workspace of its own with its schedule in it, then the same rotation is timed.
    wss = [torch.empty(ra.rollout_attn_workspace_size(dec.ctx, d.c), dtype=torch.uint8, device="cuda:0") for d in devs]
    for d, w in zip(devs, wss):
        ra.rollout_attn_decode(dec.ctx, d.set(flags).c, ctypes.c_void_p(w.data_ptr()), w.numel(), sp)
        d.set(flags | ra.RA_FLAG_REUSE_SCHEDULE)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        k = i % len(devs)
        ra.rollout_attn_decode(dec.ctx, devs[k].c, ctypes.c_void_p(wss[k].data_ptr()), wss[k].numel(), sp)
    stream.synchronize()
    reuse_wall = time.perf_counter() - t0
    out["schedule_reused"] = {"ms_per_step": round(reuse_wall * 1e3 / args.steps, 5),
                              "GBps": round(total_bytes / reuse_wall / 1e9, 1),
                              "note": "the same rotation with RA_FLAG_REUSE_SCHEDULE on a schedule computed once per instance, as "
                                      "the layers of a model after the first would call it (the attention workgroups take the "
                                      "lists they kept instead of planning again); `value` always includes the schedule"}
    for d in devs:
        d.set(flags)
    del wss

    # Two independent batches taking turns on two streams (two contexts, two workspaces; even and odd steps of the same
    # rotation): a step's planning pass and the thinning out at its end run under the other stream's page stream.  Not
    # what `value` measures (one stream, as one model's decode steps come), reported beside it.
    if len(devs) % 2 == 0 and not args.no_extras:
        dec2 = ra.Decoder(0)
        two = [(dec, torch.cuda.Stream(0)), (dec2, torch.cuda.Stream(0))]      # default priority
        for i in range(2 * len(devs)):
            two[i % 2][0].decode(devs[i % len(devs)].c, two[i % 2][1])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            two[i % 2][0].decode(devs[i % len(devs)].c, two[i % 2][1])
        torch.cuda.synchronize()
        two_wall = time.perf_counter() - t0
        out["two_streams"] = {"ms_per_step": round(two_wall * 1e3 / args.steps, 5), "GBps": round(total_bytes / two_wall / 1e9, 1),
                              "note": "the same steps issued alternately on two streams by two contexts (an instance always on "
                                      "the same stream): independent batches overlap each other's planning and tail"}
        dec2.close()

    # instance 0's result for the parity check at the end, taken before anything below writes to the pools
    dec.decode(devs[0].c, stream)
    gpu_out0, gpu_lse0 = devs[0].results()

    if not args.child:
        # The KV append that precedes each decode step's attention, timed on its own (it is not part of `value`):
        # all-zero rows, written past the ends of the sequences.  (Where the instances share one pool under different
        # block tables, these rows can land on pages that another instance reads; nothing is measured on them afterwards.)
        zero_rows = torch.zeros(probs[0].B, probs[0].Hkv, probs[0].D, dtype=torch.bfloat16, device="cuda:0")
        for _ in range(10):
            dec.append(devs[0].c, zero_rows, zero_rows, stream)
        ev0.record(stream)
        for i in range(100):
            dec.append(devs[i % len(devs)].c, zero_rows, zero_rows, stream)
        ev1.record(stream)
        torch.cuda.synchronize()
        out["append"] = {"us_per_call": round(ev0.elapsed_time(ev1) * 10, 2), "tokens_per_call": probs[0].B,
                         "note": "one token per sequence, all kv heads; launch-bound"}

        # The prompt prefill that precedes the first decode step (not part of `value` either): the workload's prompts, one
        # per group, causal attention on the matrix cores plus the write of their K/V rows into pages of instance 0's pool
        # layout.  Algorithmic operations: 4 D per (query, key) pair under the causal mask and per head.
        del zero_rows
        if cfg["prompt"] > 0:            # (a workload without prompts has no prefill to time)
            pb = workload.make_prefill(args.workload, seed=0)
            pq, pk, pv = (bits_to_bf16(x, "cuda:0") for x in (pb.q, pb.k, pb.v))
            pcu = torch.from_numpy(pb.cu_seqlens).to("cuda:0")
            pout = torch.empty_like(pq)
            plse = torch.empty(pq.shape[:2], dtype=torch.float32, device="cuda:0")
            kpool = torch.empty((pb.num_pages, pb.Hkv, 16, pb.D), dtype=torch.bfloat16, device="cuda:0")
            vpool = torch.empty_like(kpool)
            poff, ppages = torch.from_numpy(pb.page_offsets).to("cuda:0"), torch.from_numpy(pb.pages).to("cuda:0")
            pf_att = ra.prefill_from_tensors(pq, pk, pv, pcu, int(pb.lens.max()), pout, plse, float(pb.softmax_scale))
            pf_all = ra.prefill_from_tensors(pq, pk, pv, pcu, int(pb.lens.max()), pout, plse, float(pb.softmax_scale), k_pool=kpool,
                                             v_pool=vpool, page_offsets=poff, pages=ppages)
            pf_us = []
            for desc in (pf_att, pf_all):
                for _ in range(5):
                    dec.prefill(desc, stream)
                ev0.record(stream)
                for _ in range(20):
                    dec.prefill(desc, stream)
                ev1.record(stream)
                torch.cuda.synchronize()
                pf_us.append(ev0.elapsed_time(ev1) * 1e3 / 20)
            pf_tflops = pb.flops() / pf_us[0] / 1e6
            out["prefill"] = {"us_per_call": round(pf_us[1], 1), "attention_us": round(pf_us[0], 1), "prompts": int(pb.lens.size),
                              "prompt_len": int(pb.lens[0]), "algorithmic_GFLOP": round(pb.flops() / 1e9, 2),
                              "roofline": {"bound": "mfma", "kernel": "prefill_kernel", "achieved": round(pf_tflops, 1), "peak": 2500.0,
                                           "unit": "TFLOP/s", "frac": round(pf_tflops / 2500.0, 4), "traffic": None},
                              "note": "causal attention of the prompts (bf16 MFMA, fp32 accumulation); us_per_call includes the cache write"}
            del pq, pk, pv, pout, plse, kpool, vpool

    if not args.no_cpu_baseline:
        import oracle
        reps = 3
        t0 = time.perf_counter()
        for _ in range(reps):
            ref_out, ref_lse = oracle.decode(probs[0])
        cpu = (time.perf_counter() - t0) / reps
        out["cpu_baseline"] = {"value": round(alg_bytes[0] / cpu / 1e9, 3), "unit": "GB/s", "cores": oracle.threads(),
                               "kind": "oracle", "steps_per_s": round(1 / cpu, 3),
                               "sample": "all %d (sequence, head) rows of instance 0, %d repetitions, fp64 C oracle with OpenMP"
                                         % (probs[0].B * probs[0].Hq, reps)}
        # and on one thread: one (sequence, head) row in eight of the same instance
        rows = np.arange(0, probs[0].B * probs[0].Hq, 8, dtype=np.int32)
        t0 = time.perf_counter()
        oracle.decode(probs[0], rows=rows, nthreads=1)
        one = (time.perf_counter() - t0) * (probs[0].B * probs[0].Hq / rows.size)
        out["cpu_baseline"]["one_thread"] = {"value": round(alg_bytes[0] / one / 1e9, 4), "unit": "GB/s", "steps_per_s": round(1 / one, 4),
                                             "sample": "every eighth (sequence, head) row of instance 0 on one thread, scaled to all rows"}
        # the timed GPU result of instance 0 must agree with what was just computed
        errs = row_errors(gpu_out0, gpu_lse0, ref_out, ref_lse)
        assert errs[0] <= 1e-2 and errs[1] <= 1e-2 and errs[2] <= 1e-3, "bench instance 0 disagrees with the oracle: %s" % (errs,)
        out["parity"] = {"max_abs": float("%.3g" % errs[0]), "max_row_rel": float("%.3g" % errs[1]), "max_lse": float("%.3g" % errs[2])}
    out.update(extras)
    print(json.dumps(out))


def consecutive_steps(args, cfg, name, dec, stream, flags):
    """The streaming configuration as it runs: its consecutive decode steps one after the other over a static pool;
    before every step the harness uploads that step's lengths, block table (re-drawn), prefix page list and queries
    (timed separately), then the step runs with its schedule rebuilt (it is part of every call)."""
    import numpy as np
    import torch
    import paper_2507_01663_amd as ra
    import workload
    from paper_2507_01663_amd.torch_util import DeviceProblem, bits_to_bf16
    nsteps = cfg["steps"]
    width = (cfg["prompt"] + cfg["resp_max"] + nsteps) // 16 + 1
    t0 = time.time()
    p0 = workload.make_problem(args.workload, seed=0, step=0, kv_dtype=args.kv_dtype)
    pool = (p0.k_pool, p0.v_pool, p0.k_scale, p0.v_scale)
    host = []
    for st in range(nsteps):
        p = p0 if st == 0 else workload.make_problem(args.workload, seed=0, step=st, kv_dtype=args.kv_dtype, make_values=False, pool=pool,
                                                      num_pages=p0.num_pages)
        bt = np.full((p.B, width), -1, dtype=np.int32)
        bt[:, :p.block_table.shape[1]] = p.block_table
        q = p.q if p.q is not None else workload.normal_bf16(p.B * p.Hq * p.D, 0, 1000 + st).reshape(p.B, p.Hq, p.D)
        host.append(dict(bt=torch.from_numpy(bt).pin_memory(), lens=torch.from_numpy(p.seq_lens).pin_memory(),
                         pfx=torch.from_numpy(p.prefix_pages).pin_memory(),
                         q=torch.from_numpy(np.ascontiguousarray(q).view(np.int16)).pin_memory(),
                         alg=p.algorithmic_bytes(share_prefix=True)))
    p0.block_table, p0.max_pages_per_seq = host[0]["bt"].numpy(), width
    dp = DeviceProblem(p0, flags=flags)
    print("# %d steps of %s generated in %.1f s" % (nsteps, args.workload, time.time() - t0), file=sys.stderr)

    def upload(h):
        dp.block_table.copy_(h["bt"], non_blocking=True)
        dp.seq_lens.copy_(h["lens"], non_blocking=True)
        dp.pfx_pages.copy_(h["pfx"], non_blocking=True)
        dp.q.view(torch.int16).copy_(h["q"], non_blocking=True)

    ra.rollout_attn_set_timing(dec.ctx, True)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3 * nsteps)]
    for rep in range(2):                               # the first pass over the steps warms up
        phase = np.zeros((nsteps, 3))
        for st in range(nsteps):
            ev[3 * st].record(stream)
            upload(host[st])
            ev[3 * st + 1].record(stream)
            dec.decode(dp.c, stream)
            ev[3 * st + 2].record(stream)
            phase[st] = ra.rollout_attn_get_timing(dec.ctx)
        torch.cuda.synchronize()
    ra.rollout_attn_set_timing(dec.ctx, False)
    up = np.array([ev[3 * s].elapsed_time(ev[3 * s + 1]) for s in range(nsteps)])
    step = np.array([ev[3 * s + 1].elapsed_time(ev[3 * s + 2]) for s in range(nsteps)])
    alg = np.array([h["alg"] for h in host], dtype=np.float64)
    gbps = alg.sum() / (step.sum() * 1e-3) / 1e9
    att_gbps = alg.sum() / (phase[:, 1].sum() * 1e-3) / 1e9
    out = {
        "metric": "decode_attn_hbm_GBps", "value": round(gbps, 1), "unit": "GB/s", "n_gpus": 1, "steps": nsteps, "warmup": nsteps,
        "ms_per_step": round(float(step.mean()), 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if args.kv_dtype == "bf16" else "fp8_e4m3 KV, bf16 MFMA", "data": "synthetic",
        "steps_per_s": round(1e3 / float(step.mean()), 1), "pct_of_hbm_peak": round(100 * gbps / HBM_PEAK_GBPS, 2),
        "config": {"workload": name, "B": p0.B, "Hq": p0.Hq, "Hkv": p0.Hkv, "D": p0.D, "page": 16, "prefix_sharing": not args.no_sharing,
                   "algorithmic_MB_per_step": round(float(alg.mean()) / 1e6, 2)},
        "consecutive_steps": {"steps": nsteps, "total_ms": round(float(step.sum()), 4), "median_ms": round(float(np.median(step)), 5),
                              "min_ms": round(float(step.min()), 5), "max_ms": round(float(step.max()), 5),
                              "table_upload_total_ms": round(float(up.sum()), 4), "table_upload_median_ms": round(float(np.median(up)), 5),
                              "note": "every step: HIP events around the upload of its lengths, block table, prefix list and queries from "
                                      "pinned memory, then around rollout_attn_decode (schedule rebuilt in every call); the upload "
                                      "is not part of value"},
        "phases_ms": {"schedule": round(float(phase[:, 0].mean()), 5), "attention": round(float(phase[:, 1].mean()), 5),
                      "merge": round(float(phase[:, 2].mean()), 5)},
        "roofline": {"bound": "hbm", "kernel": "attention_kernel", "achieved": round(att_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(att_gbps / HBM_PEAK_GBPS, 4), "traffic": recorded_traffic(name)},
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
