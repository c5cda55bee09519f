"""MI355X-native paged decode attention with partial-output / log-sum-exp merging.

``binding`` holds the ctypes front end of the HIP library (loaded on first
use; it raises if the library has not been built).  ``workloads`` holds the
seeded synthetic input generators and imports nothing else from the package.
"""
__all__ = ["binding", "workloads"]
