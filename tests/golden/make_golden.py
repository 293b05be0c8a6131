"""Writes the stored expected values under tests/golden/.  Calls only the seeded input
generator and the CPU oracle; nothing from the HIP path.

    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import pa_oracle  # noqa: E402
from paper_2605_06068_amd import workloads  # noqa: E402


def main():
    b = workloads.make_config(1)
    out = pa_oracle.decode_batch(b, want_f64=True)["out_f64"].reshape(-1, b.head_dim)
    np.savetxt(os.path.join(HERE, "config1_seed1001_out.txt"), out, fmt="%.17e",
               header="float64 oracle output, tiny config (batch 2, 4 q heads, 2 KV heads, head_dim 64, "
                      "context_lens [37,100]), seed 1001; rows = (sequence, head), written by make_golden.py")


if __name__ == "__main__":
    main()
