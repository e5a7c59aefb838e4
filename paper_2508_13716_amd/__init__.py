"""MI355X-native partition-local layer step of cache-assisted full-batch GNN training.

The package holds three things and nothing else:

* ``csrc/``      hand-written HIP kernels for gfx950 and the C-ABI around them
                 (declared in ``include/capgnn.h`` at the repository root);
* ``binding``    a ctypes binding with the same names as the C entry points
                 (argument marshalling only, every step runs in the HIP library);
* ``synth``      seeded synthetic partitions / features / models that feed both the
                 HIP path and the CPU oracle (no arithmetic of the method lives there).

Importing the package does not load the shared library; ``binding.lib()`` does and
raises if it has not been built (``python -m paper_2508_13716_amd.build``).
"""

__all__ = ["binding", "synth", "build"]
