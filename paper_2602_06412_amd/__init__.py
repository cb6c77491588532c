"""MI355X-native SureLock hot path: thin Python binding over libsurelock.so.

Importing the package loads nothing; ``paper_2602_06412_amd.binding`` opens the
C-ABI library on first use and raises if it has not been built.
"""
__all__ = ["binding", "workloads", "build"]
