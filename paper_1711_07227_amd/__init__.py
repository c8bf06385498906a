"""LC-RWMD (linear-complexity Relaxed Word Mover's Distance) hot path for MI355X.

The compute lives in a C-ABI shared library built from `csrc/` (hand-written HIP
for gfx950); `binding` is the argument-marshalling layer over it and `synth`
draws the seeded synthetic inputs.  Nothing is imported eagerly so that the input
generator can be used without the device library.
"""
__all__ = ["binding", "synth", "build"]
