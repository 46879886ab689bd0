"""MI355X-native SVGD all-particle update (hand-written HIP behind a C ABI).

`paper_2306_06528_amd.svgd` is the Python binding of the C-ABI library; it
raises at import time if the built library is missing.  `workloads` holds the
seeded synthetic input generators and none of the method's arithmetic.
"""
__all__ = ["svgd", "workloads"]
