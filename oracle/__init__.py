"""CPU oracle for the LQER / L2QER quantized linear layer (arXiv 2402.02446).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, fp64/int64 numpy
statement of what the method computes.  It shares no code with the HIP library
and must never be imported by the product path; only the test-suite, the
smoke check and the benchmark's ``cpu_baseline`` leg may use it.

Modules
-------
mxint    MXINT block quantizer / dequantizer / canonical byte packing (Sec. 2.2, Sec. 4.1)
factors  offline construction: W_q, E_q, calibration of S, SVD split (Sec. 3.1, 3.2, App. A)
forward  the inference pass Y = X_q W_q + (X_q A_k) B_k (Eq. 3, Eq. 6)
intq     the scaled-integer variant (Table 2 "L2QER-INT": INT4 g128 weights, INT8 per-token activations)

Parity status: the paper prints no bit-level MXINT example, so the *reading*
of the format (exponent = floor(log2 amax), 1 sign + 1 integer + (b-2) fraction
bits, round-half-even, symmetric saturation, no exponent bump) is
"parity unpinned" against the authors' own numbers, and so is the reading of
the INT formats in intq (symmetric codes, FP16 scales of amax / qmax); everything
else is pinned by the tests in tests/test_oracle_*.py.
"""
