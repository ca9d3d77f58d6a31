"""MI355X-native MixLoRA feed-forward block (forward, backward, auxiliary loss).

The package holds the HIP/C-ABI library under ``csrc/``, the thin Python
binding in ``binding.py`` (argument marshalling only) and the seeded synthetic
input recipes in ``synth.py``.  Importing the package loads nothing native;
``binding.load()`` does, and raises if the library has not been built.
"""

__all__ = ["binding", "synth"]
