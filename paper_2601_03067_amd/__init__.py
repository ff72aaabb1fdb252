"""kvfuse: MI355X-native Fast Fusion (joint encoding of paged KV-cache blocks).

The compute path is the HIP library ``libkvfuse.so`` (built from ``csrc/``) behind the C ABI
declared in ``include/kvfuse.h``; ``binding`` marshals arguments to it and nothing else.  There
is no CPU fallback: importing ``binding`` without the built library raises.
``workloads`` holds the seeded synthetic input generators.
"""
__all__ = ["workloads", "binding", "build"]
