"""MI355X-native DASGD/SGNS worker step (TensAIR, arXiv 2211.10280, Algorithm 1).

The package holds four things and nothing else:

* ``csrc/``      hand-written HIP kernels for gfx950 and the C-ABI host code
                 (built into ``libtensair.so`` by ``build.py``),
* ``binding``    a thin ctypes layer with the same call names as the C ABI,
* ``trainer``    the sequence of calls of one simulated worker (no arithmetic),
* ``workload``   seeded synthetic input generators (plain data, no method
                 arithmetic), shared by tests, bench and the CPU oracle's tests.

Importing the package loads nothing native; ``binding.lib()`` loads the shared
library on first use and raises if it is missing.
"""

__all__ = ["binding", "workload", "build"]
