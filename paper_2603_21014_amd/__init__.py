"""MI355X-native cross-layer-transcoder (CLT) training step.

`paper_2603_21014_amd.binding` loads libclt.so (hand-written HIP kernels behind
a C ABI, see include/clt.h) and raises if it has not been built:
`python -m paper_2603_21014_amd.build` builds it in-tree with hipcc for gfx950.
"""
