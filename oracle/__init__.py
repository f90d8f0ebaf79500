"""CPU oracle for the Pipe-SGD aggregation + update path.

TEST INFRASTRUCTURE ONLY: imported by tests/, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  The product package never
imports this, and this package never imports the product.
"""
from .ref import *  # noqa: F401,F403
