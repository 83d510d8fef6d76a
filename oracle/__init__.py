"""float64 CPU oracle for the M2RNN recurrence -- TEST INFRASTRUCTURE ONLY.

Only the tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares nothing with the GPU library.
"""
from .m2rnn_oracle import build, fwd, bwd, num_threads  # noqa: F401
