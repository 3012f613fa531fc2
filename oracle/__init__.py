"""CPU oracle for the Ocean SpGEMM path.  TEST INFRASTRUCTURE ONLY.

Nothing under this directory is part of the product: only the tests, the
smoke check and the benchmark's ``cpu_baseline`` leg may import it.  It shares
no code with the HIP library and never imports it.
"""
