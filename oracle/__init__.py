"""CPU oracle for the sparse-residual-compensated quantized matrix multiply.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this package:
only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` do.  It shares no code with the HIP library and never imports it.
"""
