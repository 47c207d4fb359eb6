"""CPU oracle of the LVSpec verify-step hot path.  TEST INFRASTRUCTURE ONLY.

Imported by tests/, by ``__graft_entry__.smoke()`` and by the ``cpu_baseline`` leg of
``bench.py``; never by the product package.  See ``lvspec_oracle.c`` for what is computed and
which passages of the paper each function follows.
"""
from .lvspec_oracle import *  # noqa: F401,F403
