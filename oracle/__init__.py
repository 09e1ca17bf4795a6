"""Float64 CPU oracle for the eOptShrinkQ block-compression path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
package; only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline``
leg of ``bench.py`` use it.  It shares no code with the HIP library.
"""
from .eoq_oracle import *  # noqa: F401,F403
