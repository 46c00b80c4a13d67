"""ConEF per-worker hot path for MI355X (gfx950): hand-written HIP kernels behind a C ABI.

`workloads` holds the synthetic inputs; `binding` is the thin ctypes face of libconef.so
and is imported lazily so that input generation works without the compiled library.
"""
