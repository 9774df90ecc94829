"""Plain fp64 CPU oracle for the multi-adapter LoRA apply.

Test infrastructure only: imported by ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py``.  The product package never imports it.
"""
