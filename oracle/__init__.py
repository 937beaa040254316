"""CPU oracle for the Guardian fenced-kernel path.

TEST INFRASTRUCTURE ONLY.  Nothing here is part of the product: only tests/,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import it.  It shares no code with the HIP library and never imports it.

Two halves:

* ``oracle.host_model`` -- plain Python integers: partition carving, the
  partition bounds table, mask derivation, the bitwise fence, the modulo
  definition of the same fence, the copy range check and a naive first-fit
  allocator model.
* ``oracle.kernels`` -- ctypes binding of ``oracle/gd_oracle.c``: every kernel's
  semantics as one sequential loop per logical element over a simulated
  byte-addressable pool, floating point in fp64.

Parity status: every function is pinned by the CPU tests (printed example of
Section 4.3, brute force on tiny pools, equality with the modulo definition,
textbook NumPy routines on in-bounds inputs) EXCEPT the values left at
locations that a kernel's own wrapped stores alias with its own live data:
the paper leaves them unspecified (Section 4.3 only says that an offending
kernel may damage its own data), so they are "parity unpinned" and the tests
exclude them.
"""
