"""CPU oracle of the encrypted-convolution hot path.  TEST INFRASTRUCTURE ONLY.

Plain C (he_oracle.c, built with gcc) plus thin numpy client code.  Nothing in the HIP
package imports this; only tests, the smoke check and the benchmark's cpu_baseline leg do.
"""
