"""CPU oracle of the WAGMA-SGD hot path: test infrastructure, not product code.

Only ``tests/``, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package; it imports nothing from the GPU package.
"""
