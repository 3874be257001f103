"""MI355X-native scoring pass of A-RIDE (DistRL, arXiv 2410.14803).

The product is the C-ABI library built from csrc/ (declared in include/aride.h); this
package holds its thin ctypes binding (`binding`) and the seeded synthetic workload
generators (`synth`).  Importing the package loads nothing; `binding.lib()` loads the
shared library and raises if it has not been built.
"""
__all__ = ["binding", "synth"]
