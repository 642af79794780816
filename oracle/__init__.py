"""CPU oracle of the BSR step: TEST INFRASTRUCTURE ONLY (see bsr_oracle.c).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
"""
from .binding import Oracle, build_oracle, token_schedule  # noqa: F401
