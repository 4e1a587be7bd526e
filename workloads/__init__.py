"""Seeded synthetic input generators shared by the tests, the smoke check and the benchmark.

Not part of the product package: the library takes device pointers from its caller and never
draws inputs itself.  Nothing here imports the HIP binding or the CPU oracle.
"""
