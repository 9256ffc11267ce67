"""MI355X-native encoder task and embedding hand-off (HIP kernels behind a C ABI).

``workloads`` draws seeded synthetic inputs; ``binding`` marshals arguments into
``libcornenc.so``.  Nothing here computes on the CPU: without the built library
and a GPU the binding raises.
"""
