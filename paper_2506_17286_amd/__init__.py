"""MI355X-native GTA (Grouped-head latenT Attention, arXiv 2506.17286) attention forward pass.

The product is the C-ABI library built from csrc/ (gta_prefill, gta_decode, gta_cache_append);
`binding` is a thin ctypes layer over it.  Importing the package does not load the library.
"""
__all__ = ["binding", "workloads", "costmodel"]
