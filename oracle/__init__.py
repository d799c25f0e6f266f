"""CPU oracle for the tile-centric overlapped tensor-parallel operators.

TEST INFRASTRUCTURE ONLY.  Nothing under this directory is part of the product
path: only the tests, the smoke check and the benchmark's CPU-baseline leg may
import it.  It shares no code with the HIP library and never imports it.
"""
