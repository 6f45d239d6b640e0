"""MI355X-native IWDFT K/V-cache path of FAEDKV (arxiv 2507.20030).

`binding` wraps the C ABI of libiwdft.so (include/iwdft.h) one-to-one; `workload`
holds the seeded synthetic input recipes (shapes and distributions only, no
arithmetic of the method).  Importing the package does not load the library;
the first call does, and fails loudly if it has not been built.
"""
from . import workload  # noqa: F401

__all__ = ["binding", "workload", "build"]
