"""MI355X-native forward-propagation convolution (after maxDNN, arXiv 1501.06633).

The product is the C-ABI library ``libmdnn.so`` (hand-written HIP kernels for
gfx950) declared in ``include/mdnn.h``; :mod:`paper_1501_06633_amd.binding`
marshals arguments to it and nothing more.  Importing this package loads
nothing: the shared object is opened on the first call, and a missing library
is an error, never a fallback.
"""
__all__ = ["binding", "workloads"]
