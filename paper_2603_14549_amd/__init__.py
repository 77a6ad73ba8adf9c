"""MI355X-native pruning stage of ASAP (attention-shift-aware visual-token pruning).

`binding` wraps the C-ABI library (libasap.so, hand-written HIP for gfx950);
`synth` makes seeded synthetic inputs.  Importing the package loads nothing
native; `binding.load()` does, and fails loudly when the library is missing.
"""
__all__ = ["binding", "synth"]
