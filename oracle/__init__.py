"""CPU oracle for the STAR group-synchronous parameter update.

Test infrastructure only: imported by tests/, by ``__graft_entry__.smoke()`` and
by the ``cpu_baseline`` leg of ``bench.py``.  The GPU library never imports it.
"""
