"""Writes c1_tiny_fp32_oracle.txt: the fp64 oracle's outputs for configuration C1 (seeded synthetic input from
paper_2508_08192_amd.workloads.make_config(0); 1 request, 7-node binary tree, 4 query heads on 1 KV head, head_dim 64,
prefix 128).  Calls only the oracle and the input generator, never the HIP path.

    python tests/golden/write_c1_fixture.py

The file guards the oracle against silent drift: tests/test_oracle_pins.py recomputes it and compares.
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))

import oracle  # noqa: E402
from paper_2508_08192_amd import workloads as W  # noqa: E402


def main():
    w = W.make_config(0)
    out, lse = oracle.tree_attn_oracle(w.q, w.k_cache, w.v_cache, w.page_table, w.seq_lens, w.tree_parent, scale=w.scale)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_tiny_fp32_oracle.txt")
    with open(path, "w") as f:
        f.write("# oracle outputs for %s, written by write_c1_fixture.py; hexadecimal doubles\n" % w.name)
        f.write("# out[b][node][head][d] then lse[b][head][node], C order\n")
        f.write("out %d %d %d %d\n" % out.shape)
        f.write("\n".join(float(x).hex() for x in out.ravel()) + "\n")
        f.write("lse %d %d %d\n" % lse.shape)
        f.write("\n".join(float(x).hex() for x in lse.ravel()) + "\n")
    print(path)


if __name__ == "__main__":
    main()
