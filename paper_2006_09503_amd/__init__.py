"""MI355X-native 2BW pipeline-stage hot path (PipeDream-2BW, Section 3.1).

`synth` holds seeded input generators; `binding` is the ctypes layer over the C-ABI
library built from `csrc/`.  Importing the package loads nothing native; `binding`
raises if the HIP library has not been built.
"""
