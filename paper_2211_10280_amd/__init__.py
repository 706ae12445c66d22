"""MI355X-native DASGD/SGNS worker step (TensAIR, arXiv 2211.10280, Algorithm 1).

The package holds three things and nothing else:

* ``csrc/``      hand-written HIP kernels for gfx950 and the C-ABI host code
                 (built into ``libtensair.so`` by ``build.py``),
* ``binding``    a thin ctypes layer with the same call names as the C ABI,
* ``trainer``    the sequence of calls of one simulated worker (no arithmetic).

The seeded synthetic input generators (``workload.py`` at the repository root: plain
data, no method arithmetic) belong neither to this package nor to the CPU oracle;
both sides are fed from them, so the repository root must be on ``sys.path`` for the
trainer (tests, ``bench.py`` and ``__graft_entry__`` put it there).

Importing the package loads nothing native; ``binding.lib()`` loads the shared
library on first use and raises if it is missing.
"""

__all__ = ["binding", "trainer", "build"]
