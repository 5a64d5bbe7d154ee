"""GELO obfuscated QKV projection for MI355X (gfx950).

The compute path is the C-ABI library built from `csrc/` (see `include/gelo.h`);
`binding` is a thin ctypes layer over it, `workloads` generates synthetic inputs.
Nothing here falls back to a CPU implementation: using the library without the
built HIP shared object raises.
"""
