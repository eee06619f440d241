"""MI355X-native hot path of Hop (heterogeneity-aware decentralized training).

`hop` is the ctypes binding of the C-ABI library (csrc/ -> libhop.so); `inputs`
makes the seeded synthetic workloads.  Importing the package loads nothing; the
first call into `hop` loads the library and fails loudly if it is not built.
"""
