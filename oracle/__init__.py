"""CPU oracle for the SoD2 hot path -- TEST INFRASTRUCTURE, not a product path.

Plain, slow, readable re-statement of what the paper's method computes: Rank
and Dimension Propagation (Section 4.1, Alg. 1), RDP-based fusion grouping
(Section 4.2), static execution planning (Section 4.3), the peak-first arena
plan (Section 4.4.1) and the unfused operator-by-operator execution of the
graph in float64.  It shares no code with the HIP library and must only be
imported by tests, the smoke check and the CPU-baseline leg of the benchmark.
"""
