"""TEST INFRASTRUCTURE ONLY: the CPU oracle for the BitTrain bitmap codec.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The product package never does.
"""
