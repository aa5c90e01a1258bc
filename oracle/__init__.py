"""CPU oracle -- test infrastructure only.

Nothing under this package is a product path: only ``tests/``, the smoke check
and the benchmark's ``cpu_baseline`` leg may import it.  It shares no code with
``paper_2603_08734_amd`` and imports nothing from it.
"""
