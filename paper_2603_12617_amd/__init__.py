"""liboco: the per-round update of the online-ensemble learner (Sec. 3.3) as
hand-written HIP kernels for gfx950 behind a C ABI.

`workloads` draws the seeded synthetic streams; `binding` is the thin ctypes
layer over liboco.so (loaded on first use; it raises if the library has not
been built)."""
