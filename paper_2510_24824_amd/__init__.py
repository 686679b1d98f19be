"""MI355X-native Cross-Loop-Parallel decode path of the Parallel Loop Transformer.

`paper_2510_24824_amd.binding` loads the C-ABI library (libplt.so, hand-written HIP for gfx950)
and exposes its entry points under the same names; `paper_2510_24824_amd.synth` makes the
seeded synthetic inputs.  Nothing is loaded at package import time.
"""
