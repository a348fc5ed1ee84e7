"""Writes tests/golden/cfg1_seed0_expected.txt from the CPU oracle (and nothing else).

The paper prints no numeric example of attention, so there is no value of the paper's to store.  This file
freezes what the pinned oracle returns for the tiny benchmark config, so that a later edit of the oracle or of
the workload generator that moves any output is noticed.  Run from the repository root:
    python tests/golden/make_expected.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import jo  # noqa: E402
from paper_2604_23838_amd import workloads as W  # noqa: E402


def main():
    w = W.gen_config(1, 0)
    out = jo.decode_attention(w.q, w.k_pages, w.v_pages, w.block_table, w.seq_lens)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg1_seed0_expected.txt")
    with open(path, "w") as f:
        f.write("# oracle output of workloads.gen_config(1, 0): request, head, then the first 8 and last 2 of the 64\n")
        f.write("# fp32 values as hex bit patterns, and the fp64 sum of the whole row\n")
        for b in range(out.shape[0]):
            for h in range(out.shape[1]):
                row = out[b, h]
                bits = [f"{int(x):08x}" for x in np.concatenate([row[:8], row[-2:]]).view(np.uint32)]
                f.write(f"{b} {h} {' '.join(bits)} {float(row.astype(np.float64).sum())!r}\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
