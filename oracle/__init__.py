"""CPU oracle for Cyclic Data Parallelism training.  TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 numpy code written from the paper's equations and schedule.
It shares no code with the HIP library and is imported only by ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``.
The product path never calls it.
"""
