"""MI355X-native blockwise NF4 dequantisation (hand-written HIP for gfx950).

The compute lives in csrc/ behind the C-ABI declared in include/nf4.h;
`binding` marshals torch tensors into those calls.  Importing the package
does not load the library; the binding loads it on first use and raises if it
has not been built.
"""
__all__ = ["binding", "synth", "build"]
