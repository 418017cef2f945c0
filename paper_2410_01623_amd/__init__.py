"""MI355X-native Fira optimizer step (arXiv 2410.01623, Algorithm 1): C-ABI library + thin binding.

`paper_2410_01623_amd.fira` is the Python binding over the HIP library (argument marshalling
only); `paper_2410_01623_amd.synth` draws the seeded synthetic inputs.  Importing this package
does not load the HIP library; the binding loads it on first use and raises if it is missing.
"""
__all__ = ["synth"]
