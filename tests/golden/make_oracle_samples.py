"""Writes tests/golden/oracle_cfg1_samples.txt from the CPU oracle alone.

A guard against silent changes to the oracle's arithmetic: a few outputs of the
smallest workload (fp32, B=1, heads=4, d=32, 14x14 grid, 3x3 DWConv, seed 0),
computed by oracle.forward (Eq. 3 / Eq. 8 / Eq. 9 of the paper).
Run from the repo root:  python tests/golden/make_oracle_samples.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2211_10526_amd import inputs  # noqa: E402

wl = inputs.WORKLOADS[0]
x = inputs.make_inputs(wl)
out = oracle.forward(*(inputs.to_f64(x[n]) for n in ("q", "k", "v", "w")), None,
                     wl.grid_h, wl.grid_w).reshape(-1)
idx = np.linspace(0, out.size - 1, 24).astype(np.int64)
with open(os.path.join(ROOT, "tests", "golden", "oracle_cfg1_samples.txt"), "w") as f:
    f.write("# flat index into out[B,heads,N,d] and oracle.forward value; workload %s\n" % wl.name)
    f.write("# written by tests/golden/make_oracle_samples.py (calls only oracle/)\n")
    for i in idx:
        f.write("%d %.17g\n" % (i, out[i]))
