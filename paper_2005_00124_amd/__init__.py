"""MI355X-native hot path of WAGMA-SGD (arXiv 2005.00124).

``wagma``     thin ctypes binding of the C-ABI library ``libwagma.so`` built from ``csrc/``.
``workloads`` seeded synthetic inputs (shapes of the paper's models).

Importing the package loads nothing; ``wagma.load()`` raises if the HIP
library has not been built — there is no CPU fallback.
"""
