"""MI355X-native (gfx950) vectorized CNN layer path: thin Python binding over the C-ABI library.

`paper_1501_07338_amd.vcnn` mirrors the C entry points one to one; `paper_1501_07338_amd.workloads`
describes the seeded synthetic networks.  Importing the package does not load the HIP library; the
first call into `vcnn` does, and raises if it has not been built.
"""
__all__ = ["vcnn", "workloads", "net"]
