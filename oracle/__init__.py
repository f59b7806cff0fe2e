"""CPU oracle for the FedAttn attention path (fp64).

TEST INFRASTRUCTURE: imported only by tests, the smoke check and the
benchmark's CPU-baseline leg.  It shares nothing with the GPU library.

Two independent routes to the same numbers:
  * `attend_rows`, `attend_block`, `decode_step`: the row-by-row C program
    (fedattn_oracle.c), usable at every size on sampled rows;
  * `dense.*`: brute force in numpy, materialising the full L x L visibility
    matrix, for tiny inputs.
`schedule.run_stack` walks the blocks in the order of Algorithm 1.

Parity pins: every function here is pinned by tests/test_oracle_pins.py
except the two conventions the paper does not fix (GQA head grouping order,
and which of the two decode visibility readings a deployment uses); both are
listed as "parity unpinned by the paper" in the design notes, and both are
still cross-checked against brute force.
"""
from .rowwise import (attend_block, attend_rows, build, decode_step, is_sync_block,
                      n_threads, expand_keep_chunks)
from . import dense, schedule
from .aggregate import aggregate_kv

__all__ = ["attend_block", "attend_rows", "build", "decode_step", "is_sync_block",
           "n_threads", "expand_keep_chunks", "dense", "schedule", "aggregate_kv"]
