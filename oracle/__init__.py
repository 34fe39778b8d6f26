"""CPU oracle -- TEST INFRASTRUCTURE, not part of the product path.

Breadth-first (layer-by-layer) execution of a stack of non-convolution CNN
layers, as Section 3.1 / Figure 2 of the paper describes standard frameworks
doing it.  Only tests, the smoke check and the benchmark's CPU-baseline leg
import this package; the HIP library and its binding never do.
"""
