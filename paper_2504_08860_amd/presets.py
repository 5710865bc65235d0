"""Hand-picked block sizes for the five benchmark workloads: rows x columns per block and rounds
per batch, nothing else.  The library chooses these three by itself when they are left at 0
(hbp.h); bench.py reports the hand-picked values next to that choice as the "tuned_block_sizes"
leg, to show what the choice costs."""
from __future__ import annotations

TUNED = {
    1: dict(rows_per_block=512, cols_per_block=4096, rounds_per_batch=8),
    2: dict(rows_per_block=512, cols_per_block=32768, rounds_per_batch=9),
    3: dict(rows_per_block=2048, cols_per_block=32768, rounds_per_batch=4),
    4: dict(rows_per_block=2048, cols_per_block=32768, rounds_per_batch=4),
    5: dict(rows_per_block=2048, cols_per_block=32768, rounds_per_batch=4),
}


def tuned_block_sizes(config_number: int, dtype: str = "f32") -> dict:
    """Block sizes for workload ``config_number``; ``dtype`` "f64" halves the block width (the vector
    segment of a block column has to fit the same 128 KB of LDS)."""
    p = dict(TUNED[config_number])
    if dtype == "f64":
        p["cols_per_block"] = min(p["cols_per_block"], 16384)
    return p
