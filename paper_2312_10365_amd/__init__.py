"""MI355X-native routed FFN of SPT (arXiv 2312.10365): HIP kernels behind a C ABI.

`paper_2312_10365_amd.spt`    ctypes binding of libspt.so (the product path)
`paper_2312_10365_amd.inputs` seeded synthetic workloads (no method arithmetic)
`paper_2312_10365_amd.build`  hipcc build of csrc/ into libspt.so
"""
