"""MI355X-native collisionless embedding table (hot path of arxiv 2209.07663, section 2.1).

`paper_2209_07663_amd.binding` is the thin ctypes layer over the C-ABI library built from `csrc/`;
`paper_2209_07663_amd.synth` draws the seeded synthetic workloads.
"""
