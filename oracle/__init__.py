"""CPU oracle for the packed variable-length attention path.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  The product package never
imports it, and it never imports the product package.
"""
