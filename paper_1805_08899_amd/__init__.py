"""Additive (MLP) attention with the tanh feature map recomputed in the
backward pass, hand-written for MI355X (gfx950).

The compute lives in csrc/ behind the C ABI declared in include/echoattn.h;
`binding` marshals arguments to it and nothing else.  Importing the package
does not load the shared library; `binding.lib()` does, and raises if it has
not been built.
"""
__all__ = ["binding", "workloads", "footprint"]
