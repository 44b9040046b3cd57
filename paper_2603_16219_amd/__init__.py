"""MI355X-native verify-and-recover block of SpecSteer's Draft-Verify-Recover protocol.

``binding`` wraps the C-ABI HIP library (``libspecsteer.so``, built from
``csrc/``); ``workloads`` holds the seeded synthetic input recipes.  Importing
the package loads neither torch nor the library.
"""

__all__ = ["binding", "workloads"]
