"""Writes tests/golden/oracle_digests.json from the CPU oracle alone.

The paper prints no worked numeric example of threshold splitting, the
quantizer or Algorithm 1, so there are no printed values to store.  What is
stored instead are digests of the oracle's own output on the seeded synthetic
workloads, as a regression guard: a later change to the oracle's arithmetic
must change this file in the same commit and say why.

Run from the repository root:  python tests/golden/make_golden.py
This script calls only oracle/ (and the input generator).
"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import tsq_oracle as O              # noqa: E402
from paper_2511_04002_amd import synth          # noqa: E402

CASES = [
    # name, generator kwargs, dtype, tau, bit set, budget, mode
    ("C1_eps0.05", ("C1", {}), O.F16, 6.0, (2, 4, 8), 0.05, O.BUDGET_REL_RMS),
    ("C1_eps0.1", ("C1", {}), O.F16, 6.0, (2, 4, 8), 0.1, O.BUDGET_REL_RMS),
    ("C1_lsb0.2", ("C1", {}), O.F16, 6.0, (2, 4, 8), 0.2, O.BUDGET_LSB),
    ("C2_256_eps0.2", ("C2", {"tokens": 256}), O.F16, 8.0, (2, 3, 4, 6, 8), 0.2, O.BUDGET_REL_RMS),
    ("C4_1024_eps0.05", ("C4", {"tokens": 1024}), O.BF16, 10.0, (2, 3, 4, 5, 6, 8), 0.05,
     O.BUDGET_REL_RMS),
]


def digest(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def run_case(case):
    name, (wl, kw), dt, tau, bs, bud, mode = case
    x = synth.make(wl, **kw)
    c = O.compress(x, dt, tau, bs, bud, mode, nthreads=4)
    y = O.decompress(c, nthreads=4)
    return {
        "input": digest(x), "tokens": int(x.shape[0]), "hidden": int(x.shape[1]),
        "width_hist": np.bincount(c.bits, minlength=9).tolist(),
        "nnz": c.nnz, "payload_bytes": c.payload_bytes,
        "compressed_bytes": O.compressed_bytes(c),
        "bits": digest(c.bits), "scale": digest(c.scale), "pay_off": digest(c.pay_off),
        "row_ptr": digest(c.row_ptr), "payload": digest(c.payload),
        "out_col": digest(c.out_col), "out_val": digest(c.out_val), "decoded": digest(y),
    }


def main():
    out = {case[0]: run_case(case) for case in CASES}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_digests.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1, sort_keys=True)
        f.write("\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
