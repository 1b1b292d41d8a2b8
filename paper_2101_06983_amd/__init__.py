"""MI355X-native Gradient Cache hot path (arXiv 2101.06983).

`binding` mirrors the C ABI of include/gradcache.h; `synth` holds the seeded
input generators.  The compute lives in libgradcache.so (HIP, gfx950).
"""
from . import synth  # noqa: F401
from . import binding  # noqa: F401
