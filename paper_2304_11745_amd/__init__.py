"""MI355X-native multi-tenant regulated executor (GACER's hot path).

``binding`` exposes the C ABI of ``include/gacer.h`` one to one (ctypes, argument marshalling
only); ``harness`` allocates device memory and streams with PyTorch and fills the descriptor
structs.  All computation happens inside ``libgacer.so``; there is no fallback path.
"""
