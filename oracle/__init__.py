"""CPU oracle for the speculative-decoding hot path (test infrastructure only).

Plain, slow NumPy (float64) implementations of what the hot path computes:
Algorithm 1 (SpeculativeDecodingStep), the standardised sampling of section
2.2, the closed forms of section 3, and the reference transformer decoders
the synthetic workloads use.  Nothing here is imported by the product
package; only tests, the smoke check and the benchmark's cpu_baseline leg
may call it.  It shares no code with the HIP kernels.
"""
