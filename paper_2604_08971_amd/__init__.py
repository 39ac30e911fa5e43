"""MI355X-native pruned multimodal encoder forward (SentryGate + SentryAttend).

Importing the package loads nothing heavy: `workloads` is numpy-only input
generation, `binding` loads the HIP shared library on first use and raises if
it has not been built.
"""
__all__ = ["workloads", "binding"]
