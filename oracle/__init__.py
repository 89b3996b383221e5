"""CPU oracle for the FeF-DLLM speculative verify step.

TEST INFRASTRUCTURE ONLY.  Everything under ``oracle/`` is a plain, slow, fp64 numpy
statement of what the verify step computes, written from the paper (Algorithm 2, the
residual-distribution equation of the Algorithm appendix, Section 2.2, Theorems 1-2).
It shares no code with the HIP path and must never be imported by the product package;
only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may use it.
"""
