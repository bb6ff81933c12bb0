"""Seeded synthetic inputs for the KV-slab decode-attention path.

``gen`` is the host (numpy) generator, ``device`` drives the identical HIP
generator.  Nothing in this package performs any step of the method itself.
"""
from . import gen  # noqa: F401
