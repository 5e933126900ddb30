"""MI355X-native batched candidate-suffix attention over one shared prefix K/V.

The package holds only what the hot path needs:

* ``csrc/``     HIP kernels for gfx950 and the C-ABI entry points declared in ``include/pskv.h``
* ``binding``   thin ctypes marshalling layer with the same names as the C-ABI
* ``build``     in-tree hipcc build of ``libpskv.so``
* ``inputs``    seeded synthetic workload generators (data only, no attention arithmetic)

Nothing here imports the CPU oracle, and the binding raises if the HIP library is missing.
"""

__all__ = ["binding", "build", "inputs"]
