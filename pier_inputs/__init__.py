"""Seeded synthetic inputs shared by the tests, the smoke run and the benchmark:
workload shapes (shapes.py), the host generator (generator.py) and its device
twin (device.py + csrc/pier_inputs.hip).  None of the optimizer's arithmetic."""
