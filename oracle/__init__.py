"""float64 CPU oracle for the M2RNN recurrence and for the scan's two neighbours in the block
-- TEST INFRASTRUCTURE ONLY.

Only the tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares nothing with the GPU library.
"""
from . import m2rnn_block_oracle as block  # noqa: F401
from . import m2rnn_oracle
from .m2rnn_oracle import fwd, bwd, num_threads  # noqa: F401


def build(force=False):
    """Compile both C oracles with gcc."""
    m2rnn_oracle.build(force)
    block.build(force)
