"""MI355X-native batched egocentric voxel-world renderer (RGB uint8 + depth float32 for every
agent camera of thousands of voxel environments per step) behind a five-call C ABI.

``binding`` marshals arguments into ``libmv.so`` (hand-written HIP for gfx950); ``synth`` draws the
seeded synthetic workloads; ``build`` compiles the library in-tree.
"""
from . import binding, synth  # noqa: F401
from .binding import Batch, MvError, PinnedBuffer, load_library  # noqa: F401
