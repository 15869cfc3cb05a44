"""CPU oracle for the Quaff quantized-linear hot path.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the HIP product path never does.  `oracle.api` wraps the plain-C
implementation in `quaff_oracle.c` with numpy arrays.
"""
