"""MI355X-native blockwise-distillation hot path (teacher relay + student steps).

`workloads` holds descriptors and seeded inputs (pure data, no GPU needed);
`pbd` is the ctypes binding over the HIP library and fails loudly when the
library has not been built.
"""
