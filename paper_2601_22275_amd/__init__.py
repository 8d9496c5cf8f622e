"""MI355X-native spatio-temporal Monarch attention (VMonarch hot path).

The compute lives in ``csrc/`` (hand-written HIP for gfx950 behind a C ABI,
declared in ``include/vmonarch.h``).  ``binding`` marshals arguments for the
library; ``synth`` builds the seeded synthetic workloads.
"""
