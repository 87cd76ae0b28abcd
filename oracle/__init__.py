"""CPU oracle of the verification step: test infrastructure, not product code.

Plain, slow, float64 numpy written from the paper's definitions.  Only the
tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the HIP path shares no code with it and never calls it.
"""
