"""fp64 CPU oracles of the LSM recurrence (diagonal decays, delta rule) -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the GPU library.
"""
from .lsm_oracle import (  # noqa: F401
    KIND_NONE, KIND_HEAD, KIND_SCALAR, KIND_VECTOR,
    build_oracle, oracle_threads, lsm_oracle_fwd, lsm_oracle_bwd,
)
from .delta_oracle import build_delta_oracle, delta_oracle_fwd, delta_oracle_bwd  # noqa: F401
