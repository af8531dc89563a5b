"""MI355X-native BitDelta hot path: 1-bit delta compressor and multi-tenant linear (arxiv 2402.10193).

The compute lives in libbitdelta.so (hand-written HIP for gfx950, C ABI in include/bitdelta.h);
`binding` marshals torch tensors into that ABI and `synth` draws seeded synthetic inputs.
"""
from . import synth  # noqa: F401

__all__ = ["binding", "synth", "build"]
