"""MI355X-native implementation of FREE's parallel verification pass.

`paper_2511_20390_amd.binding` is the ctypes binding over the C-ABI library
(hand-written HIP for gfx950); `paper_2511_20390_amd.synth` holds the seeded
synthetic-input generators.  Importing the package loads nothing native: the
library is opened on first use and its absence is an error, never a fallback.
"""
