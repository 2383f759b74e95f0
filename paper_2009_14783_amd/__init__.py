"""MI355X-native (gfx950) implementation of one worker's share of a HetSeq training step.

`paper_2009_14783_amd.binding` is the thin ctypes layer over the C-ABI library
(`libhetseq_hip.so`, declared in include/hetseq_hip.h); `paper_2009_14783_amd.synth`
draws seeded synthetic inputs.  Importing this package loads nothing native: the
library is loaded on first use of the binding and a missing library is an error.
"""
