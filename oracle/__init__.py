"""CPU oracle of the DSSD verification step (test infrastructure, not a product path).

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  See dssd_oracle.cpp for what is computed and which passages it follows.
"""
