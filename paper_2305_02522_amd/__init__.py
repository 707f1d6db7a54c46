"""MI355X-native binary GNN inference (bit-pack, adjacency build, XNOR-popcount
BGEMM, bit-SpMM with fused threshold/re-pack) behind a C-ABI library.

`paper_2305_02522_amd.binding` loads `libbitgnn.so` (built in-tree by
`paper_2305_02522_amd.build`) and raises if it is missing: there is no CPU
fallback.  `paper_2305_02522_amd.workloads` only generates seeded inputs.
"""
__all__ = ["binding", "workloads", "build"]
