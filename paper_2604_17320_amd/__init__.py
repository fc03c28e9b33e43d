"""MI355X-native W4A4 prefill layer with in-layer visual-token pruning (QUOTA hot path).

The compute lives in ``csrc/`` (hand-written HIP for gfx950 behind a C ABI,
declared in ``include/quota.h``).  ``binding`` marshals torch device pointers
into that ABI; ``workloads`` generates the seeded synthetic inputs.
"""
__all__ = ["binding", "workloads", "build"]
