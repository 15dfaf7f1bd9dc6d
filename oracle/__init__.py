"""CPU oracle for the HLQ backward pass -- TEST INFRASTRUCTURE.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares nothing with the HIP library
(``paper_2406_15102_amd``) and neither imports the other.
"""
from .hlq_oracle import *  # noqa: F401,F403
