"""Writes tests/golden/tiny_decode_oracle.json from the CPU oracle alone.

The paper prints no numerical example of attention, so no golden value can be the
paper's; this file only freezes what the pinned oracle returns on the seeded tiny
decode configuration, so that an accidental change to the oracle or to the input
generator is noticed.  Run from the repository root:  python tests/golden/make_golden.py
"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
import workloads as W  # noqa: E402


def main() -> None:
    w = W.tiny_decode()
    out = oracle.attention(w.geom, w.pool, w.q, w.block_tables, w.seq_lens, w.scale, nthreads=1)
    rec = {
        "source": "oracle.attention on workloads.tiny_decode() (seed 20251101); not a value from the paper",
        "seq_lens": [int(x) for x in w.seq_lens],
        "rows": {"%d,%d" % (r, h): [float.hex(float(x)) for x in out[r, h, :8]] for r in (0, 3, 7) for h in (0, 3)},
    }
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_decode_oracle.json"), "w") as f:
        json.dump(rec, f, indent=1)


if __name__ == "__main__":
    main()
