"""CPU oracle for the MoE layer forward (test infrastructure only).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the HIP library and
imports nothing from the product package.
"""
from .moe_oracle import (  # noqa: F401
    ACT, DTYPE, Oracle, build_oracle, load_oracle, oracle_lib_path,
)
