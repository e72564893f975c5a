"""CPU oracle for the conv hot path: TEST INFRASTRUCTURE ONLY.

A slow, plain float64 statement of what the weight transformations and the
convolution kernels must compute, written from the mathematics (zero-padded
cross-correlation; Cook-Toom construction of the Winograd F(m x m, 3 x 3)
matrices) and pinned by the tests under tests/ that carry no `gpu` marker.

Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may
import this package.  It shares no code with the GPU library and the GPU
library never calls it.

Parity pins per function are listed in each module's header.
"""
