"""MI355X-native sequence-tiled LM-head projection + cross-entropy (forward and backward).

`paper_2506_13996_amd.binding` wraps the C-ABI library built from `csrc/`; `synth` draws the
seeded synthetic inputs.  Importing the package does not load the HIP library; the binding
loads it on first use and raises if it has not been built.
"""
__all__ = ["binding", "synth"]
