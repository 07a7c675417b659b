"""Writes tests/golden/tiny_seed0.json from the oracle alone (never from the HIP path).

The paper prints no numeric example for decode attention, so this file is not
a pin of the oracle's arithmetic (tests/test_oracle_pins.py does that with
closed forms and brute force); it freezes the Tiny configuration's inputs and
oracle results so that an accidental change to the generator or the oracle
shows up as a diff.  Run:  python tests/golden/make_golden.py
"""
import hashlib
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle      # noqa: E402
import workload    # noqa: E402


def record(kv_dtype):
    p = workload.make_problem("tiny", seed=0, kv_dtype=kv_dtype)
    out, lse = oracle.decode(p)
    h = hashlib.sha256()
    for a in (p.q, p.k_pool, p.v_pool, p.block_table, p.seq_lens):
        h.update(a.tobytes())
    return {"inputs_sha256": h.hexdigest(), "seq_lens": p.seq_lens.tolist(),
            "block_table_row0": p.block_table[0].tolist(),
            "lse": [[x.hex() for x in row] for row in lse.tolist()],
            "out_b3_h0_first8": [x.hex() for x in out[3, 0, :8].tolist()]}


if __name__ == "__main__":
    data = {"source": "oracle.decode on workload.make_problem('tiny', seed=0); values are C99 hex floats",
            "bf16": record("bf16"), "fp8_e4m3": record("fp8_e4m3")}
    with open(os.path.join(HERE, "tiny_seed0.json"), "w") as f:
        json.dump(data, f, indent=1)
    print("wrote tiny_seed0.json")
