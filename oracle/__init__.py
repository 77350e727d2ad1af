"""CPU oracle of the WindowQuant hot path: test infrastructure only.

Nothing in the GPU package imports this; it is used by ``tests/``, by the smoke
check and by the benchmark's ``cpu_baseline`` leg.
"""
