"""libuncomp: UNComp's prefill-time KV-cache compression pass as hand-written
HIP kernels for gfx950 behind a C ABI, plus this thin ctypes binding.

``paper_2410_03090_amd.binding`` loads the shared library (and raises if it has
not been built); ``paper_2410_03090_amd.synth`` generates the seeded inputs.
"""
__all__ = ["binding", "synth"]
