"""CPU oracle for the LAMPS decode hot path (arXiv 2410.18248).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  The product package never
imports it, and it never imports the product package.

``attention``  -- Section 2.2 equation, fp64, over logical un-paged K/V
                  (C source in ``lamps_oracle.c``).
``blocks``     -- byte-exact model of the Swap / Discard / Preserve handling
                  strategies (Section 1, Section 4.2) on a block pool.
``cache``      -- the logical KV cache growing by one position per iteration
                  (Section 2.2.1), for the append step.
``scheduler``  -- equations (1)-(3), the memory-over-time rank and Algorithm 1
                  as a plain iteration-level simulation.
"""
from .attention import build, decode_attn, max_threads, prefill_attn, widen  # noqa: F401
from .blocks import AllocatorModel, PoolModel, kv_bytes_per_token  # noqa: F401
from .cache import LogicalCache  # noqa: F401
from . import scheduler  # noqa: F401
