"""CPU oracle for the data-tiering hot path.  TEST INFRASTRUCTURE ONLY.

Nothing under this folder is part of the product: only tests, the smoke check
and the benchmark's ``cpu_baseline`` leg may import it, and it imports nothing
from the GPU package.
"""
