"""CPU oracle for the kvtrim hot path (TEST INFRASTRUCTURE ONLY).

Thin ctypes binding over ``kvtrim_oracle.c`` plus a host-side ragged cache
container.  Nothing here imports or is imported by the HIP path; only tests,
the smoke check and the benchmark's ``cpu_baseline`` leg may use it.
"""
from .host import (Gate, HostCache, Shape, build, gate_forward, lib, score, score_horizon, select, compact, attend, append, occupancy,
                   key_of_score, set_threads, threads)

__all__ = ["Gate", "gate_forward", "HostCache", "Shape", "build", "lib", "score", "score_horizon", "select", "compact",
           "attend", "append", "occupancy", "key_of_score", "set_threads", "threads"]
