"""CPU oracle of the Balanced-Sparsity hot path: TEST INFRASTRUCTURE ONLY.

Only ``tests/``, the smoke check and the bench's ``cpu_baseline`` leg may import
this package; the product package never does.
"""
