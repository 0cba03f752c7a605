"""Writes tests/golden/config1_oracle.txt from the CPU oracle alone.

Run from the repo root:  python tests/golden/make_golden.py
The file guards against silent drift of the oracle or of the seeded generator;
it is not an independent pin (those live in tests/test_oracle_pins.py).
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from taper_inputs import fill_values_numpy, structure_config1  # noqa: E402


def main():
    b = fill_values_numpy(structure_config1())
    st, sh = b.structure, b.structure.shape
    out, lse, _, _ = oracle.attention(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.page_size, sh.scale, b.q, b.kv,
                                      st.block_table, st.prefix_len, st.suffix_len)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config1_oracle.txt")
    with open(path, "w") as f:
        f.write("# tiny workload (4 q heads, 1 kv head, D 64, page 16; serial 256 + prefix 192 x suffixes 0/8/17/32)\n")
        f.write("# written by tests/golden/make_golden.py from oracle/ only; columns: seq head lse out[0] out[21] out[63]\n")
        for s in range(st.n_seqs):
            for h in range(sh.n_q_heads):
                f.write(f"{s} {h} {lse[s, h]:.17g} {out[s, h, 0]:.17g} {out[s, h, 21]:.17g} {out[s, h, 63]:.17g}\n")
        f.write("# block table rows (first 18 entries)\n")
        for s in range(st.n_seqs):
            f.write("bt " + " ".join(str(int(x)) for x in st.block_table[s, :18]) + "\n")


if __name__ == "__main__":
    main()
