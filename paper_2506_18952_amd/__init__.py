"""MI355X-native batched verify step of HOLA's Hierarchical Speculative Decoding.

``binding`` (loaded on first use) wraps the C-ABI library ``libhola.so`` built from
``csrc/``; ``workloads`` holds the seeded synthetic logit generators.
"""
__all__ = ["binding", "workloads"]
