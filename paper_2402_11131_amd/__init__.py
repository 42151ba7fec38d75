"""MI355X-native verify-and-speculate step of Speculative Streaming.

``paper_2402_11131_amd.api`` is the Python binding of ``libss.so`` (argument
marshalling only); ``paper_2402_11131_amd.synth`` draws the seeded synthetic
workloads.  Nothing is loaded at import time; the first call into ``api`` loads
the HIP library and raises if it has not been built.
"""
__all__ = ["api", "synth", "build"]
