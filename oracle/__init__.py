"""CPU oracle of the MVUE N:M prune + update-GEMM path.  TEST INFRASTRUCTURE ONLY.

Nothing under this directory is part of the product: it may be imported by the tests,
by ``__graft_entry__.smoke()`` and by the ``cpu_baseline`` leg of ``bench.py`` only.
``mvue_oracle.c`` is the step-by-step algorithm (binary32 decisions, binary64 GEMM),
``ideal.py`` the paper's formulas in exact-arithmetic form, ``cwrap.py`` the loader.
"""
