"""MI355X-native hot path of Randomized Automatic Differentiation.

`binding` is the ctypes layer over librad_hip.so (the C ABI of include/rad.h);
`synth` holds the seeded synthetic-input generators; `build` compiles the
library.  Importing this package loads nothing: `binding.lib()` does, and
fails loudly when the library has not been built.
"""
