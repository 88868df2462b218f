"""CPU oracle for the NGC eviction step and decode attention.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``.  The product package never
imports it and it never imports the product package.
"""
from .ngc_oracle import *  # noqa: F401,F403
from .paged import PagedCache  # noqa: F401
