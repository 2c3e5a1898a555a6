"""MI355X-native hot path of Astraea's token-wise attention (arXiv 2506.05096).

`binding` exposes the C ABI of libastraea (HIP kernels for gfx950); `synth`
draws the seeded synthetic workloads; `layer` chains the calls of one
layer-step on caller-owned buffers.
"""
from . import binding, synth  # noqa: F401
