"""MI355X-native KV-cache context switching: the swap hot path of FastSwitch
(arXiv 2411.18424) as hand-written HIP kernels behind a C ABI.

``paper_2411_18424_amd.kvswap`` is the binding over the shared library (it
fails loudly when the library has not been built); ``synth`` holds the seeded
synthetic workloads.  Nothing is imported eagerly so that ``synth`` can be used
on machines without the library.
"""

__all__ = ["kvswap", "synth", "build"]
