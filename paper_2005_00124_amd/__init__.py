"""MI355X-native hot path of WAGMA-SGD (arXiv 2005.00124).

``libwagma``  thin ctypes binding of the C-ABI library built from ``csrc/``.
``workloads`` seeded synthetic inputs (shapes of the paper's models).

Importing the package loads nothing; ``libwagma.load()`` raises if the HIP
library has not been built — there is no CPU fallback.
"""
