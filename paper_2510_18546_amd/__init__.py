"""MI355X-native segmented prefill attention over retrieval-selected KV segments
(the planning-step hot path of EfficientNav, arXiv 2510.18546).

Sub-modules are imported on demand: ``inputs`` (seeded synthetic workloads, no
method arithmetic), ``binding`` (ctypes binding over the C ABI of
``libefficientnav.so``) and ``build`` (hipcc build of that library).
"""

__all__ = ["inputs", "binding", "build"]
