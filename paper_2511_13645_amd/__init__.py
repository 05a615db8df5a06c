"""MI355X-native fused neighbor sampling + GraphSAGE-mean aggregation (arXiv 2511.13645).

``paper_2511_13645_amd.binding`` -- ctypes binding of the C-ABI HIP library (the product).
``paper_2511_13645_amd.synth``   -- seeded synthetic inputs (no arithmetic of the method).
Importing the package loads nothing; the HIP library is loaded on first use of the binding.
"""
__all__ = ["binding", "synth"]
