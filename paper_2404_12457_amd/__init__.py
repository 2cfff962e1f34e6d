"""ragc: prefix-cached paged prefill attention for MI355X (gfx950).

`workload` draws seeded synthetic inputs; `binding` is the thin ctypes layer
over the C-ABI library built from `csrc/`.  Importing the package loads
neither; the binding raises if the HIP library has not been built."""
