"""MI355X-native paged decode attention and KV block repack behind DP / TP layout views.

The compute lives in ``csrc/`` (HIP for gfx950, C ABI declared in ``include/flying_kv.h``);
``binding`` marshals arguments to it, ``workloads`` draws the seeded synthetic inputs.
"""
from . import workloads  # noqa: F401
