"""MI355X-native DWDP MoE-layer hot path: C-ABI HIP library plus a thin ctypes binding.

`paper_2604_01621_amd.inputs`  seeded synthetic workloads (no layer arithmetic)
`paper_2604_01621_amd.binding` ctypes wrappers named after the C entry points
`paper_2604_01621_amd.build`   hipcc build of csrc/ into libdwdp.so (in-tree)
"""
