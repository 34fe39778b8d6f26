"""MI355X-native depth-first execution of stacks of non-convolution CNN layers.

`paper_1804_08378_amd.brainslug` is the thin ctypes binding of the C-ABI HIP library
(libbrainslug_hip.so); `paper_1804_08378_amd.workloads` holds the seeded synthetic
inputs and the named stack configurations.  Importing this package loads
nothing native; the binding loads the library on first use and fails loudly if
it has not been built.
"""
__version__ = "0.1.0"
