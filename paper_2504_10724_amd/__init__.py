"""libee for AMD MI355X: the batched early-exit decode step (HELIOS, arXiv
2504.10724) as hand-written HIP kernels behind a C ABI.  `capi` is the thin
binding with the names of include/ee.h; `session` holds the PyTorch device
buffers the library borrows."""
from . import capi  # noqa: F401

__all__ = ["capi", "session", "build"]
