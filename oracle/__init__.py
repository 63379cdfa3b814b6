"""CPU oracle for the MISA indexer.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path (the HIP library and its Python binding) may
import this package; only tests, the smoke check and the benchmark's
CPU-baseline leg use it.  It shares no code with the HIP path.
"""
