"""Writes tests/golden/config1_rows.txt from the fp64 checker alone (no GPU code involved).

The paper prints no numeric worked example of attention, so nothing here is the paper's;
the file only guards the checker against silent change.  Rows: batch tokens 0, 63, 64, 65, 66
of the tiny workload (first/last chunk row and the three decodes), all heads, flattened.
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2403_02310_amd import workloads as wl  # noqa: E402

if __name__ == "__main__":
    b = wl.config1_tiny()
    toks = [0, 63, 64, 65, 66]
    out = oracle.attention_for_batch(b, tokens=toks)
    np.savetxt(os.path.join(os.path.dirname(os.path.abspath(__file__)), "config1_rows.txt"),
               out.reshape(len(toks), -1), fmt="%.17e",
               header="fp64 checker rows of workloads.config1_tiny(): tokens 0,63,64,65,66 x (4 heads x 64)")
