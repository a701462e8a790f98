"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke run.

``workloads.synth`` generates the inputs (numpy, no attention arithmetic); ``workloads.device``
moves a generated workload to the GPU.  Neither the HIP library nor the CPU oracle lives here, and
neither of them imports this package: the callers hand the same arrays to both.
"""
__all__ = ["synth", "device"]
