"""MI355X-native reduction engine of a multi-rail allreduce (Nezha, arXiv 2405.17870).

``paper_2405_17870_amd.nezha_sim`` is the thin binding over the C-ABI library
``libnezha_sim.so`` (hand-written HIP for gfx950); ``paper_2405_17870_amd.inputs``
makes the seeded synthetic workloads; ``paper_2405_17870_amd.placement`` places a
caller's buffers in chosen regions of HBM.  Importing the package does not load the
native library; the first call into ``nezha_sim`` does, and fails loudly if it
has not been built.
"""
__all__ = ["inputs", "nezha_sim", "placement"]
