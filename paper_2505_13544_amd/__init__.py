"""libmtla for MI355X: hand-written HIP kernels behind a C ABI (include/mtla.h)
for the MTLA decode hot path -- cache append/merge, absorbed decode attention
over the strided latent cache, and the stride-aware-masked prefill form.

`binding` mirrors the C entry points through ctypes; `session` adds torch
device-memory plumbing.  Importing `binding` requires the built library."""

__all__ = ["binding", "session", "build"]
