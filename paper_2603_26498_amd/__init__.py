"""MI355X (gfx950) vision preprocess + ViT-encode library: Python side.

`binding` mirrors the C ABI of include/tcmv.h one to one; `runtime` adds a small
convenience class that owns device buffers through PyTorch.  All computation
happens in libtcmv.so (hand-written HIP kernels); build it with
`python -m paper_2603_26498_amd.build`."""
from . import binding  # noqa: F401

__all__ = ["binding"]
