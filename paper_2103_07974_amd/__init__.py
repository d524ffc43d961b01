"""MI355X-native fused gradient synchronisation for CrossoverScheduler (arXiv 2103.07974).

`paper_2103_07974_amd.xs` is the ctypes binding of the HIP library;
`paper_2103_07974_amd.workloads` holds the seeded synthetic gradient sets.
Importing the package loads nothing native; the binding loads the library on first use.
"""
__all__ = ["workloads", "xs"]
