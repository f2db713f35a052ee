"""CPU oracle for the Load path of the Reuse Store (test infrastructure).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It is independent of the HIP library:
it imports nothing from the product package and the product imports nothing
from here.

Three parts:

* ``oracle.c`` (built to ``liboracle.so`` with gcc): the byte-level
  definitions -- fingerprint, bytewise equality, copy -- as scalar C loops.
* ``reuse_store.py``: the Reuse Store's bookkeeping (Tensor Mapping lookup,
  best-fit allocation over the Region List, assembly, release) as plain
  Python over lists, one linear scan per decision.
* ``pure.py``: the fingerprint again in pure Python integers, for brute-force
  checks on tiny inputs.

Parity status: every function here is pinned by ``tests/test_oracle_*.py``
(public SplitMix64 vectors, closed forms, algebraic invariants, brute force,
a hand-derived allocation example).  No function here is "parity unpinned".
"""
from .cbytes import (build_liboracle, bytes_equal, copy_bytes, fingerprint,
                     splitmix64)
from .pure import fingerprint_py, splitmix64_py
from .reuse_store import (H2D, REUSE, Entry, NoSpace, OraclePlan, PlanOp,
                          ReuseStoreOracle, StalePlan)

__all__ = [
    "build_liboracle", "bytes_equal", "copy_bytes", "fingerprint",
    "splitmix64", "fingerprint_py", "splitmix64_py", "H2D", "REUSE", "Entry",
    "NoSpace", "OraclePlan", "PlanOp", "ReuseStoreOracle", "StalePlan",
]
