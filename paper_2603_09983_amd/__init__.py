"""MI355X-native verify-step MoE layer (MoE-SpAc hot path).

`paper_2603_09983_amd.binding` loads the HIP C-ABI library and fails loudly if
it is not built; `paper_2603_09983_amd.synth` holds the seeded input recipes.
Nothing is imported eagerly here so that CPU-only tooling can use `synth`.
"""
__all__ = ["binding", "synth"]
