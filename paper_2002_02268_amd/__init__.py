"""MI355X-native fp32 matrix product (the dense GEMM of the paper's Section 6 case study).

The compute path is the HIP library under ``csrc/`` reached through a C ABI;
``binding`` marshals torch device tensors into it.  ``synth`` makes seeded inputs.
Nothing is loaded at import time; the first call into ``binding`` loads the built
library and raises if it is missing.
"""
