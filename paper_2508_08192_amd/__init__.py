"""libtreeattn: tree attention for the verification step of tree-based speculative decoding on MI355X.

`paper_2508_08192_amd.treeattn` is the thin ctypes binding of the C-ABI library built from csrc/;
`paper_2508_08192_amd.workloads` draws the seeded synthetic inputs.
"""
