"""CPU oracle for the fused-operator templates -- TEST INFRASTRUCTURE ONLY.

This package is the plain, slow, operator-at-a-time reference that the GPU
library is checked against.  It evaluates each expression the way the paper's
unfused "Base" plans do (Sec. 1 "Fusion Opportunities", Fig. 1a-1d; Sec. 5.2):
one basic operator per pass, every intermediate materialised.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import it.  It shares no code with the GPU path and never
imports it; the product must never route through it.

Modules
-------
build     compile ``oracle_ops.c`` with gcc into ``liboracle_ops.so``
ops       the basic operators (element-wise, aggregates, products)
unfused   operator-at-a-time evaluators of a symbolic postfix expression,
          one per template (Cell, MAgg, Row, Outer)
plans     the five benchmark workloads written out as explicit unfused plans
interp    a naive per-cell / per-row / per-non-zero interpreter of the same
          expressions (pure Python loops, tiny inputs): the independent
          "fused-semantics" evaluator the unfused plans are pinned against
"""
