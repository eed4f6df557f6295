"""CPU oracle for the speculative-decoding verify step.

TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64 implementations of what the hot path computes,
written from the paper's statement of the method.  Only ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py`` may import this package; the product package
never does, and this package never imports the product package.
"""
