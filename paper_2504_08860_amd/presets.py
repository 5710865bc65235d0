"""Block-parameter presets for the five benchmark workloads (R rows x C columns per block,
fixed share of the schedule).  Chosen by measurement on MI355X; the library's
own defaults are the paper's 512 x 4096."""
from __future__ import annotations

PRESETS = {
    1: dict(rows_per_block=512, cols_per_block=4096, fixed_fraction_q8=256),
    2: dict(rows_per_block=512, cols_per_block=32768, rounds_per_batch=9, fixed_fraction_q8=256, slot_weight=4, column_weight=0),
    3: dict(rows_per_block=2048, cols_per_block=32768, rounds_per_batch=4, fixed_fraction_q8=256, column_weight=50000),
    # weights from a least-squares fit of the workers' times: a range costs per group, per round and per block
    # column entered (26 us + 18 ns, 3 ns and 19 us; 0.6 ns per slot, 0.03 ns per nonzero)
    4: dict(rows_per_block=2048, cols_per_block=32768, rounds_per_batch=4, fixed_fraction_q8=240, slot_weight=18,
            group_weight=522, round_weight=89, column_weight=540000, heavy_group_rounds=4096),
    5: dict(rows_per_block=2048, cols_per_block=32768, rounds_per_batch=4, fixed_fraction_q8=256, column_weight=100000),
}


def preset(config_number: int, dtype: str = "f32") -> dict:
    """Parameters for workload ``config_number``; ``dtype`` "f64" gives those of the fp64 variant."""
    p = dict(PRESETS[config_number])
    if dtype == "f64":
        # the vector segment of a block column has to fit the same 128 KB of LDS; with twice as
        # many block columns the R-MAT matrix runs best without a competitive part
        p["cols_per_block"] = min(p["cols_per_block"], 16384)
        if config_number == 4:
            p.update(fixed_fraction_q8=256, heavy_group_rounds=2048)
        if config_number == 5:
            p["column_weight"] = 200000
    return p
