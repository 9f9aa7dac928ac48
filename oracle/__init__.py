"""CPU oracle (test infrastructure only).

Thin ctypes wrapper over ``nm_oracle.c``.  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the GPU library never does.
"""
from .oracle import *  # noqa: F401,F403
