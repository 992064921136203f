"""Early-exit LLM decode step for MI355X (gfx950): HIP kernels behind a C ABI plus a thin ctypes binding.

`paper_2407_20272_amd.binding` loads the native library; `paper_2407_20272_amd.workloads` generates the
seeded synthetic inputs.  Importing the package itself loads nothing native.
"""
