"""CPU oracle of the padding-free MoE layer.  TEST INFRASTRUCTURE ONLY: importable from tests/,
__graft_entry__.smoke() and the cpu_baseline leg of bench.py - never from the product package."""
from .moe_oracle import *  # noqa: F401,F403
