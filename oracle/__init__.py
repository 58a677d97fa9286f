"""TEST INFRASTRUCTURE: the fp64 CPU parity oracle (see gdn_oracle.c).

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package.  It never imports the HIP library or its Python binding.
"""
