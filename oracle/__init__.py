"""CPU oracle for the convolution-forward path.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the bench's ``cpu_baseline`` leg may import
this package; the HIP library and its Python binding never do, and nothing here
imports them.
"""
