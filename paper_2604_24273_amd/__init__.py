"""MI355X-native forward pass of the frozen ternary state encoder of BitRL.

`synth` draws seeded inputs; `binding` is the thin ctypes layer over the
C-ABI library built from `csrc/`.  Importing the package does not load the
library; `binding.lib()` does, and raises if it has not been built.
"""
