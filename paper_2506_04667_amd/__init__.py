"""MI355X-native forward pass of one GPU's share of a top-k MoE layer.

The arithmetic lives in the HIP library under ``csrc/`` behind the C ABI declared
in ``include/moe.h``; ``binding`` marshals arguments to it and nothing else.
Importing the package loads nothing; ``binding.load()`` fails loudly when the
built library is missing.
"""
