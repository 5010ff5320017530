"""ifx: block-causal attention against a per-layer KV cache, and the cache
commit, for the block-diffusion decode loop of the Inferix paper (arXiv
2511.20714), as hand-written HIP for MI355X (gfx950) behind a C ABI.

``binding`` mirrors the C entry points of include/ifx.h one to one (argument
marshalling only); ``build`` compiles the shared library; ``synth`` draws the
seeded synthetic inputs.  There is no CPU fallback anywhere in this package.
"""
from . import binding, build, synth  # noqa: F401
from .binding import KVCache, IFX_BF16, IFX_F32  # noqa: F401
