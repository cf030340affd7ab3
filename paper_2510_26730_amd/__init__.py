"""MI355X-native MoE-layer hot path with adaptive expert prefetching and cache-aware routing.

``binding`` exposes the C ABI of ``libexpertflow.so`` (see ``include/expertflow.h``);
``synth`` draws the seeded synthetic workloads; ``build`` compiles the library.
Importing the package loads nothing; the library is loaded on first use and its
absence is an error (there is no fallback path).
"""
__all__ = ["binding", "synth", "build"]
