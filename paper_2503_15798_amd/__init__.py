"""MoLE lookup-expert layer for MI355X (gfx950): thin Python binding over libmole.

Importing the package does not load the HIP library; `paper_2503_15798_amd.binding`
does so on first use and raises if it is missing.
"""
__all__ = ["workloads", "accounting", "binding", "build"]
