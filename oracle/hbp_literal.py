"""The paper's literal HBP layout, for tiny inputs only (TEST INFRASTRUCTURE ONLY).

Pure-Python loops, written for readability.  Every row of every block owns a slot, so
``zero_row`` and ``output_hash`` have n_rows x (number of column blocks) entries as
Section 3.1 states; blocks are numbered row-major, bm * NBC + bn, as the index formulas
of Algorithms 2 and 3 do; ``col`` holds global column indices (Algorithm 3 reduces them
modulo the block width when it reads the vector segment).

Readings of garbled or silent passages used here:
  * blocks are R rows x C columns (the text's M/N are used inconsistently);
  * slot base of block (bm, bn) is (bm * NBC + bn) * R for full row blocks; for the ragged
    last row block only real rows own slots, so bases come from a running sum;
  * rows without nonzeros in the block take part in the reorder with key(0) = 0;
  * slot order inside a block is ascending (key, local row);
  * Algorithm 3's loop accumulates first and stops when add_sign is negative (its text,
    not its ``while add_sign[j] > 0`` listing, which would drop every row's last element).
"""
from __future__ import annotations

import numpy as np


def hash_key(n: int, a: int, R: int) -> int:
    """aggregation + dispersion + linear mapping (Section 3.2), this build's reading."""
    b = max(1, R // 9)
    d = b
    c = 1 << a
    agg = min(n >> a, 8)
    lin = ((n % c) * d) >> a
    return min(agg * b + lin, R - 1)


class LiteralHbp:
    def __init__(self, ptr, col, val, n_rows, n_cols, R, C, W, a):
        self.n_rows, self.n_cols, self.R, self.C, self.W, self.a = n_rows, n_cols, R, C, W, a
        NBR = -(-n_rows // R)
        NBC = -(-n_cols // C)
        self.NBR, self.NBC = NBR, NBC
        self.output_hash, self.zero_row = [], []
        self.begin_ptr, self.begin_nnz, self.slot_base = [], [], []
        self.col, self.data, self.add_sign = [], [], []
        for bm in range(NBR):
            rows = range(bm * R, min((bm + 1) * R, n_rows))
            for bn in range(NBC):
                lo, hi = bn * C, (bn + 1) * C
                # Algorithm 2: the row's nonzeros inside this column block
                seg = {}
                for r in rows:
                    js = [j for j in range(ptr[r], ptr[r + 1]) if lo <= col[j] < hi]
                    seg[r - bm * R] = js
                order = sorted(seg, key=lambda q: (hash_key(len(seg[q]), a, R), q))
                self.slot_base.append(len(self.output_hash))
                self.begin_nnz.append(len(self.col))
                for g0 in range(0, len(order), W):
                    lanes = order[g0:g0 + W]
                    self.begin_ptr.append(len(self.col))
                    zeros_before = 0
                    for q in lanes:
                        self.output_hash.append(q)
                        if len(seg[q]) == 0:
                            self.zero_row.append(-1)
                            zeros_before += 1
                        else:
                            self.zero_row.append(zeros_before)
                    # column-major fill with the running count of rows still being stored
                    remaining = {q: len(seg[q]) for q in lanes}
                    live = sum(1 for q in lanes if remaining[q] > 0)
                    k = 0
                    while live > 0:
                        for q in lanes:
                            if k < len(seg[q]):
                                j = seg[q][k]
                                self.col.append(int(col[j]))
                                self.data.append(float(val[j]))
                                remaining[q] -= 1
                                if remaining[q] == 0:
                                    self.add_sign.append(-1)
                                    live -= 1
                                else:
                                    self.add_sign.append(live)
                        k += 1
        self.begin_ptr.append(len(self.col))
        self.begin_nnz.append(len(self.col))
        self.slot_base.append(len(self.output_hash))

    def spmv(self, x):
        """Two-step SpMV: per-block partial vectors (Algorithm 3), then the combine part.
        Returns (y, partials) with partials[bm][bn] a list over local rows; fp64."""
        R, C, W = self.R, self.C, self.W
        partials = [[None] * self.NBC for _ in range(self.NBR)]
        group = 0
        for bm in range(self.NBR):
            n_local = min(R, self.n_rows - bm * R)
            for bn in range(self.NBC):
                blk = bm * self.NBC + bn
                base = self.slot_base[blk]
                vect = [float(x[c]) if c < self.n_cols else 0.0 for c in range(bn * C, (bn + 1) * C)]
                out = [0.0] * n_local
                for i in range(0, n_local, W):          # one group at a time
                    for q in range(min(W, n_local - i)):  # lane q
                        slot = base + i + q
                        if self.zero_row[slot] == -1:
                            out[self.output_hash[slot]] = 0.0
                            continue
                        j = self.begin_ptr[group] + q - self.zero_row[slot]
                        s = 0.0
                        while True:
                            s += self.data[j] * vect[self.col[j] % C]
                            step = self.add_sign[j]
                            if step < 0:
                                break
                            j += step
                        out[self.output_hash[slot]] = s
                    group += 1
                partials[bm][bn] = out
        y = np.zeros(self.n_rows, dtype=np.float64)
        for bm in range(self.NBR):
            for bn in range(self.NBC):
                for q, v in enumerate(partials[bm][bn]):
                    y[bm * R + q] += v
        return y, partials
