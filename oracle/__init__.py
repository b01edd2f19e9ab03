"""CPU oracle of the CD-SGD hot path.  TEST INFRASTRUCTURE, NOT THE PRODUCT.

Import only from tests, the smoke check and the benchmark's cpu-baseline leg.
"""
