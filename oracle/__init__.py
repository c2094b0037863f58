"""CPU oracle for the eXmY codec: test infrastructure only.

Nothing in the product package may import this; only ``tests/``, the smoke
check and the ``cpu_baseline`` leg of ``bench.py`` do.
"""
