"""Decode under a concurrent host-to-device weight copy (the device-visible side of the paper's delayed parameter
update, Sec. 5.2, where new weights stream to the rollout workers while they generate): `bench.py --weight-copy`
queues pinned-memory copies on a second stream of default priority for the whole of the timed steps.  This runs a short
version in a process of its own and checks what the record in profiles/weight_copy_interference.md relies on: the copies
outlast the steps, both rates are real, and the steps still run at a sensible fraction of their undisturbed rate."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def bench(*flags):
    cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "150", "--warmup", "20", "--no-cpu-baseline", "--no-extras"] + list(flags)
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    return json.loads([l for l in r.stdout.splitlines() if l.startswith("{")][-1])


def test_decode_while_weights_stream_in():
    quiet = bench()
    busy = bench("--weight-copy")
    wc = busy["weight_copy"]
    print("undisturbed %.1f GB/s; with copies %.1f GB/s; host to device %.1f GB/s over %d copies" % (
        quiet["value"], busy["value"], wc["host_to_device_GBps"], wc["copies"]), flush=True)
    assert wc["copy_seconds"] >= wc["steps_seconds"], "the copies ended before the timed steps did"
    assert wc["host_to_device_GBps"] > 5.0                      # a PCIe link, not a stalled stream
    assert 0.5 * quiet["value"] < busy["value"] <= 1.05 * quiet["value"]
    assert "weight_copy" not in quiet
