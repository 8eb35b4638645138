"""MI355X-native sequence-scheduling decode path.

Sub-modules are imported on demand so that the seeded input generator
(``synth``) can be used without loading the HIP library:

* ``synth``   - seeded synthetic workloads and weights (inputs only).
* ``binding`` - ctypes binding of the C-ABI library ``libss.so``.
* ``build``   - compiles ``csrc/`` for gfx950 into ``libss.so``.
"""

__all__ = ["synth", "binding", "build"]
