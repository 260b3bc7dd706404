"""CPU oracle of the ESPO hot path.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this package.  The GPU product path never does.
"""
from .espo_oracle import (  # noqa: F401
    OracleParams,
    build_oracle,
    gae_bruteforce,
    advantages,
    advantages_packed,
    advantages_terminal,
    batch_stats,
    gumbel,
    gumbel_at,
    block_draw,
    num_threads,
    philox4x32_10,
    set_threads,
    state_update,
    step,
    stream_word,
    uniform,
    whiten,
)
