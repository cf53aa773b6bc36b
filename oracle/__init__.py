"""CPU oracle for sparse graph attention -- TEST INFRASTRUCTURE, not product code.

`reference` is the dense NumPy definition (small L); `rowscan` is the
row-sampled C version for problems too large for a dense L x L matrix.  Only
tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the HIP product path never does.
"""
