"""MI355X-native hot path of Tempo's memory-reduced Transformer layers.

`workloads` (seeded synthetic inputs) imports nothing heavy; `binding` loads the HIP
shared library and fails loudly when it has not been built.
"""
__all__ = ["binding", "workloads"]
