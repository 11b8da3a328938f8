"""MI355X-native shard of a tensor-parallel transformer layer (arXiv 1909.08053, Section 3).

The compute path is the HIP library built from ``csrc/`` and loaded by
``paper_1909_08053_amd.binding``; importing this package loads nothing heavy.
"""
__all__ = ["synth", "binding", "pipeline", "build"]
