"""COMP-AMS optimizer step for MI355X (gfx950): hand-written HIP kernels behind a C ABI.

`binding` loads the shared library and marshals arguments; `workloads` holds the
seeded synthetic inputs.  There is no CPU fallback: without the built library the
binding raises.
"""
