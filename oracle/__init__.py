"""CPU oracle for the SFC hot path (test infrastructure, not product code).

Everything under this package is a plain, slow, fp64/int64 numpy statement of
what the paper's method computes.  It exists so that tests can check the HIP
library against it; only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import it.  It shares no code, table
or constant with the HIP path and never imports it.
"""
