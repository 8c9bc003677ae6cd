"""h1bkv: MI355X (gfx950) decode attention over a 1-bit-key / 4-bit-value KV cache (arxiv 2510.05529).

`binding` is the thin ctypes layer over the C-ABI library built from csrc/ (include/h1bkv.h);
`workloads` holds the seeded synthetic inputs.  Nothing is imported eagerly so that the package
can be imported on a machine where the library has not been built yet.
"""
__all__ = ["binding", "workloads", "build"]
