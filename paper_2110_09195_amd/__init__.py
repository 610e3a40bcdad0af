"""MI355X-native sub-bit binary 3x3 convolution (Sub-bit Neural Networks, arXiv 2110.09195).

The product is the C-ABI HIP library declared in include/snn.h; `binding` is its thin
ctypes wrapper and `synth` the seeded input generators.  Importing the package does not
load the library; `binding.lib()` does, and fails loudly if it has not been built.
"""
