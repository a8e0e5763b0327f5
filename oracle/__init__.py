"""CPU fp64 oracle of the TSR-Adam per-matrix path.  TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import this
package; the GPU library never does.  `tsr_oracle` wraps the plain C implementation,
`accounting` holds the paper's byte and memory formulas.
"""
