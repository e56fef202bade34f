"""MI355X (gfx950) implementation of the IMPACT learner's hot path (arXiv 1912.00167).

The work is done by hand-written HIP kernels in ``libimpact.so`` behind the C ABI
declared in ``include/impact.h``.  ``binding`` is a thin ctypes layer with the same
entry-point names: it only marshals arguments (PyTorch is used for device memory
and streams).  Importing this package does not load the library; the first call
does, and fails loudly when it has not been built.
"""

__all__ = ["binding", "build"]
