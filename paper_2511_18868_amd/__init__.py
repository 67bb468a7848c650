"""MI355X-native arm-scoring pass of a KernelBand search round.

`synth` draws seeded inputs and has no GPU dependency.  Everything else goes
through the C-ABI library built from `csrc/` (see `binding`), which is loaded on
first use and fails loudly when it is missing.
"""
__all__ = ["synth", "binding"]
