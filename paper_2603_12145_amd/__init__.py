"""MI355X-native vectorised environment step / reset / rollout.

`paper_2603_12145_amd.binding` is the thin ctypes layer over libmi355env.so (built in-tree by
`paper_2603_12145_amd.build`); `paper_2603_12145_amd.inputs` holds the seeded synthetic input
generators shared by tests and benchmarks.  Importing the package loads nothing.
"""
