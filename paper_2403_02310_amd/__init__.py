"""Hybrid-batch paged attention for MI355X (gfx950): Python binding of libsarathi.

``paper_2403_02310_amd.binding`` marshals arguments for the C ABI declared in
``include/sarathi.h``; ``paper_2403_02310_amd.workloads`` holds the seeded synthetic inputs.
Nothing is imported eagerly, so the input generators work without the built library.
"""

__all__ = ["binding", "workloads", "build"]
