"""CPU oracle for the EFIM cache-hit attention path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
package; only the tests, the smoke check and the CPU-baseline leg of the
benchmark do.  It shares no code with the HIP library.
"""
