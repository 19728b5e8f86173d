"""MI355X-native scaled-Muon optimizer step (hand-written HIP behind a C ABI).

``binding`` exposes the C entry points; ``workloads`` holds the seeded synthetic
inputs; ``build`` compiles the library in-tree for gfx950.
"""
__all__ = ["binding", "workloads", "build"]
