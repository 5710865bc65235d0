"""Pins for the oracle's HBP layout: the hand-worked example, the HBP->COO round trip,
brute-force recounts on tiny inputs, closed forms and special cases (W = 1, one block)."""
import json
import os

import numpy as np
import pytest

from oracle.hbp_literal import LiteralHbp
from workloads import make_config, random_csr, widen_to_f64, worked_example_8x8

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_8x8.json")


def build(oracle, m, **kw):
    return oracle.OracleHbp(m.ptr, m.col, m.val, m.n_rows, m.n_cols, **kw)


def coo_set(rows, cols, vals):
    bits = np.asarray(vals, dtype=np.float32).view(np.uint32).astype(np.int64)
    return sorted(zip(np.asarray(rows).tolist(), np.asarray(cols).tolist(), bits.tolist()))


def csr_coo(m):
    rows = np.repeat(np.arange(m.n_rows), np.diff(m.ptr))
    return coo_set(rows, m.col, m.val)


# ---------------------------------------------------------------- worked example

def test_worked_example_literal():
    g = json.load(open(GOLDEN))
    m = worked_example_8x8()
    L = LiteralHbp(m.ptr, m.col, m.val, 8, 8, g["R"], g["C"], g["W"], g["a"])
    lit = g["literal"]
    for name in ("output_hash", "zero_row", "begin_ptr", "begin_nnz", "col", "data", "add_sign"):
        assert list(getattr(L, name)) == lit[name], name
    y, partials = L.spmv(m.x)
    assert y.tolist() == g["y"]
    assert partials == lit["partials"]


def test_worked_example_compact(oracle):
    g = json.load(open(GOLDEN))
    m = worked_example_8x8()
    h = build(oracle, m, R=g["R"], C=g["C"], W=g["W"], hash_shift=g["a"])
    for name, want in g["compact"].items():
        if name.startswith("_") or name == "partial":
            continue
        assert h.array(name).tolist() == want, name
    y, partial = h.spmv(m.x)
    assert y.tolist() == g["y"]
    assert partial.tolist() == g["compact"]["partial"]
    sch = g["schedule"]
    h2 = build(oracle, m, R=g["R"], C=g["C"], W=g["W"], hash_shift=g["a"], num_workers=sch["P"], fixed_q8=sch["fixed_q8"])
    for name in ("col_group_ptr", "comp_lo", "comp_col", "fixed_start", "fixed_col"):
        assert h2.array(name).tolist() == sch[name], name


# ---------------------------------------------------------------- brute force helpers

def brute_segments(m, R, C):
    """{(bn, bm): [(local row, [csr positions])]} by direct definition."""
    blocks = {}
    for r in range(m.n_rows):
        per_bn = {}
        for j in range(m.ptr[r], m.ptr[r + 1]):
            per_bn.setdefault(int(m.col[j]) // C, []).append(j)
        for bn, js in per_bn.items():
            blocks.setdefault((bn, r // R), []).append((r % R, js))
    return blocks


CASES = [
    # rows, cols, density, seed, R, C, W, shift
    (40, 40, 0.2, 1, 8, 8, 4, -1),
    (77, 53, 0.3, 2, 16, 10, 4, 0),
    (64, 200, 0.15, 3, 64, 32, 8, 1),
    (129, 65, 0.5, 4, 32, 16, 3, 2),
    (30, 300, 0.4, 5, 7, 50, 64, -1),
    (200, 30, 0.1, 6, 512, 4096, 64, -1),
]


@pytest.mark.parametrize("case", CASES)
def test_layout_against_brute_force(oracle, case):
    nr, nc, dens, seed, R, C, W, shift = case
    m = random_csr(nr, nc, dens, seed, empty_row_frac=0.15)
    h = build(oracle, m, R=R, C=C, W=W, hash_shift=shift)
    a = h.a
    blocks = brute_segments(m, R, C)
    order = sorted(blocks)                                     # (bn, bm): column-major
    assert h.B == len(order) and h.nnz == m.nnz
    assert list(zip(h.array("blk_bn").tolist(), h.array("blk_bm").tolist())) == order
    slot_ptr, gptr_blk = h.array("slot_ptr"), h.array("blk_group_ptr")
    row_local, seg_len = h.array("row_local"), h.array("seg_len")
    group_ptr, group_slot = h.array("group_ptr"), h.array("group_slot")
    col_local, data, add_sign = h.array("col_local"), h.array("data"), h.array("add_sign")
    assert slot_ptr[0] == 0 and slot_ptr[-1] == h.S == sum(len(v) for v in blocks.values())
    g = 0
    for b, key in enumerate(order):
        segs = blocks[key]
        s0, s1 = slot_ptr[b], slot_ptr[b + 1]
        assert s1 - s0 == len(segs)
        # slots: ascending (hash key, local row), uniquely determined
        want = sorted(segs, key=lambda t: (oracle.hash_key(len(t[1]), a, R), t[0]))
        assert row_local[s0:s1].tolist() == [q for q, _ in want]
        assert seg_len[s0:s1].tolist() == [len(js) for _, js in want]
        assert gptr_blk[b] == g
        for w0 in range(0, len(want), W):
            lanes = want[w0:w0 + W]
            assert group_slot[g] == s0 + w0
            pos = group_ptr[g]
            # round-by-round (column-major) fill, rows keep CSR order
            for k in range(max(len(js) for _, js in lanes)):
                for li, (q, js) in enumerate(lanes):
                    if k < len(js):
                        assert col_local[pos] == m.col[js[k]] - key[0] * C
                        assert data[pos] == m.val[js[k]]
                        # closed form of add_sign: elements after it in this round plus
                        # elements before it in the next round, plus one
                        if k + 1 == len(js):
                            assert add_sign[pos] == -1
                        else:
                            after = sum(1 for _, j2 in lanes[li + 1:] if k < len(j2))
                            before = sum(1 for _, j2 in lanes[:li] if k + 1 < len(j2))
                            assert add_sign[pos] == after + before + 1
                        pos += 1
            g += 1
            assert group_ptr[g] == pos
    assert g == h.G and gptr_blk[-1] == g and group_slot[-1] == h.S and group_ptr[-1] == m.nnz
    # column index of blocks and the combine index
    cbp = h.array("col_blk_ptr")
    for bn in range(h.NBC):
        assert list(range(cbp[bn], cbp[bn + 1])) == [i for i, k in enumerate(order) if k[0] == bn]
    sp, sb = h.array("stripe_ptr"), h.array("stripe_blk")
    for bm in range(h.NBR):
        assert sb[sp[bm]:sp[bm + 1]].tolist() == [i for i, k in enumerate(order) if k[1] == bm]


@pytest.mark.parametrize("case", CASES)
def test_round_trip_and_spmv(oracle, case):
    nr, nc, dens, seed, R, C, W, shift = case
    m = random_csr(nr, nc, dens, seed, empty_row_frac=0.15)
    h = build(oracle, m, R=R, C=C, W=W, hash_shift=shift)
    assert coo_set(*h.to_coo()) == csr_coo(m)                    # exact (row, col, value bits) multiset
    y_ref, s = oracle.csr_spmv_f64(m.ptr, m.col, m.val, m.x)
    y, partial = h.spmv(m.x)
    assert np.all(np.abs(y - y_ref) <= 1e-13 * s)
    assert np.all(y[np.diff(m.ptr) == 0] == 0)


@pytest.mark.parametrize("case", CASES[:4])
def test_literal_and_compact_agree(oracle, case):
    nr, nc, dens, seed, R, C, W, shift = case
    m = random_csr(nr, nc, dens, seed, empty_row_frac=0.15)
    h = build(oracle, m, R=R, C=C, W=W, hash_shift=shift)
    L = LiteralHbp(m.ptr, m.col, m.val, m.n_rows, m.n_cols, R, C, W, h.a)
    y_lit, partials = L.spmv(m.x)
    y_ref, s = oracle.csr_spmv_f64(m.ptr, m.col, m.val, m.x)
    assert np.all(np.abs(y_lit - y_ref) <= 1e-13 * s)
    # compact slots = literal slots with the empty rows dropped, block by block
    row_local, slot_ptr = h.array("row_local"), h.array("slot_ptr")
    _, partial = h.spmv(m.x)
    for b in range(h.B):
        bm, bn = h.array("blk_bm")[b], h.array("blk_bn")[b]
        blk = bm * L.NBC + bn
        lo, hi = L.slot_base[blk], L.slot_base[blk + 1]
        kept = [L.output_hash[s] for s in range(lo, hi) if L.zero_row[s] != -1]
        assert row_local[slot_ptr[b]:slot_ptr[b + 1]].tolist() == kept
        for s in range(slot_ptr[b], slot_ptr[b + 1]):
            assert abs(partial[s] - partials[bm][bn][row_local[s]]) <= 1e-12 * max(1.0, abs(partial[s]))
    # literal array lengths the paper states: add_sign = nnz; zero_row, output_hash = rows x column blocks
    assert len(L.add_sign) == m.nnz
    assert len(L.zero_row) == len(L.output_hash) == m.n_rows * L.NBC


def test_w1_blocks_are_csr_order(oracle):
    """W = 1: a group is one row, so each block's col/data are its rows' CSR runs in slot order
    and add_sign is 1 inside a row, -1 at its end."""
    m = random_csr(90, 70, 0.25, 11, empty_row_frac=0.1)
    R, C = 16, 32
    h = build(oracle, m, R=R, C=C, W=1, hash_shift=-1)
    blocks = brute_segments(m, R, C)
    pos = 0
    for b in range(h.B):
        key = (int(h.array("blk_bn")[b]), int(h.array("blk_bm")[b]))
        by_row = dict(blocks[key])
        for s in range(h.array("slot_ptr")[b], h.array("slot_ptr")[b + 1]):
            js = by_row[int(h.array("row_local")[s])]
            assert h.array("data")[pos:pos + len(js)].tolist() == m.val[js].tolist()
            assert h.array("add_sign")[pos:pos + len(js)].tolist() == [1] * (len(js) - 1) + [-1]
            pos += len(js)
    assert pos == m.nnz


def test_single_block_equal_rows_reproduces_csr(oracle):
    """One block, W = 1, all rows equally long: the reorder is the identity and col/data are
    the CSR arrays verbatim."""
    rows, n = 25, 6
    rng = np.random.default_rng(5)
    col = np.concatenate([np.sort(rng.choice(40, n, replace=False)) for _ in range(rows)]).astype(np.int32)
    ptr = (np.arange(rows + 1) * n).astype(np.int32)
    val = rng.standard_normal(rows * n).astype(np.float32)
    h = oracle.OracleHbp(ptr, col, val, rows, 40, R=32, C=64, W=1)
    assert h.B == 1 and h.array("row_local").tolist() == list(range(rows))
    assert np.array_equal(h.array("col_local"), col.astype(np.uint16))
    assert np.array_equal(h.array("data"), val)


def test_equal_rows_any_w_is_ell(oracle):
    """All rows equally long in one block: a full group is a column-major (ELL) tile."""
    rows, n, W = 16, 5, 8
    ptr = (np.arange(rows + 1) * n).astype(np.int32)
    col = np.tile(np.arange(n), rows).astype(np.int32) * 2
    val = np.arange(rows * n, dtype=np.float32)
    h = oracle.OracleHbp(ptr, col, val, rows, 16, R=16, C=16, W=W)
    want = val.reshape(2, W, n).transpose(0, 2, 1).ravel()
    assert np.array_equal(h.array("data"), want)
    assert set(h.array("add_sign").tolist()) == {W, -1}


def test_schedule_split(oracle):
    """Section 3.3 split: the P ranges tile the group list and have equal weight up to one group;
    every range keeps the stated share of its weight fixed, up to one group, and its competitive
    tail lies inside the block column of its last group."""
    m = random_csr(300, 300, 0.05, 3)
    for P, q8, sw, gw, cw, colw in [(1, 128, 1, 0, 0, 0), (4, 192, 4, 0, 7, 0), (7, 255, 1, 9, 0, 40), (64, 256, 6, 100, 300, 0),
                                    (5, 0, 0, 1, 50, 1000), (1000, 100, 1, 0, 0, 3), (6, 256, 1, 0, 0, 100000)]:
        h = build(oracle, m, R=16, C=16, W=8, num_workers=P, fixed_q8=q8, slot_weight=sw, round_weight=gw, group_weight=cw,
                  column_weight=colw)
        assert h.P == P and h.fixed_q8 == q8
        wt = h.array("group_ptr").astype(np.int64) + sw * h.array("group_slot").astype(np.int64) + gw * h.array("group_rounds").astype(np.int64) + cw * np.arange(h.G + 1)
        cgp, comp_lo = h.array("col_group_ptr"), h.array("comp_lo")
        # the cut into ranges also charges every block column that holds a group to its first group
        starts = cgp[:-1][np.diff(cgp) > 0]
        wt_cut = wt + colw * np.array([(starts < g).sum() for g in range(h.G + 1)], dtype=np.int64)
        fs, fc = h.array("fixed_start"), h.array("fixed_col")
        assert np.array_equal(cgp, h.array("blk_group_ptr")[h.array("col_blk_ptr")])
        assert fs[0] == 0 and fs[-1] == h.G and np.all(np.diff(fs) >= 0)
        col_of = np.searchsorted(cgp, np.arange(h.G), side="right") - 1
        comp_col = h.array("comp_col")
        assert comp_lo.shape == (P,) and comp_col.shape == (P,)
        for w in range(P):
            if fs[w] < h.G:
                assert fc[w] == col_of[fs[w]]
            # equal weight: the range starts at the first group whose preceding weight reaches w/P
            assert wt_cut[fs[w]] * P >= w * wt_cut[-1]
            assert fs[w] == 0 or wt_cut[fs[w] - 1] * P < w * wt_cut[-1]
            g0, g1 = fs[w], fs[w + 1]
            assert g0 <= comp_lo[w] <= g1
            if g1 == g0:
                assert comp_col[w] == fc[w]
                continue
            last_col = col_of[g1 - 1]
            assert comp_col[w] == last_col and np.all(col_of[comp_lo[w]:g1] == last_col)
            tot = wt[g1] - wt[g0]
            share = next(g for g in range(g0, g1 + 1) if (wt[g] - wt[g0]) * 256 >= tot * q8)   # by the definition
            assert comp_lo[w] == max(share, cgp[last_col])
        if q8 == 256:
            assert np.array_equal(comp_lo, fs[1:])                 # nothing left to competition
        if q8 == 0:
            # everything of a range's last block column is competitive
            assert all(comp_lo[w] == max(fs[w], cgp[comp_col[w]]) for w in range(P) if fs[w + 1] > fs[w])
        if colw == 100000:
            # a column weighs far more than all groups: every worker's range starts at a column's
            # first group or just behind it (there the column's charge has been paid)
            first = np.isin(fs[:-1], cgp) | np.isin(fs[:-1] - 1, starts)
            assert np.all(first)


def test_group_rounds(oracle):
    """group_rounds is the running sum of the groups' longest rows (brute force from seg_len)."""
    m = random_csr(300, 500, 0.06, 5)
    h = build(oracle, m, R=16, C=32, W=8)
    seg_len, gs, gr = h.array("seg_len"), h.array("group_slot"), h.array("group_rounds")
    assert gr[0] == 0 and len(gr) == h.G + 1
    for g in range(h.G):
        assert gr[g + 1] - gr[g] == seg_len[gs[g]:gs[g + 1]].max()


def test_combine_units(oracle):
    """Combine units: every row block owns max(1, ceil(slots / unit_slots)) consecutive units that
    tile its stripe_blk range in order; a unit starts at the first entry that reaches its share of
    the row block's slots (brute force), so none holds more than that share plus one block."""
    m = random_csr(400, 900, 0.08, 11)
    for unit_slots in (64, 100, 1000, 1 << 20):
        h = build(oracle, m, R=32, C=16, W=8, unit_slots=unit_slots)
        sp, sb, slot_ptr = h.array("stripe_ptr"), h.array("stripe_blk"), h.array("slot_ptr")
        up, us, uk, ms = h.array("unit_ptr"), h.array("unit_stripe"), h.array("unit_k"), h.array("multi_stripes")
        size = (slot_ptr[1:] - slot_ptr[:-1])[sb].astype(np.int64)
        assert h.U == up[-1] == len(us) and len(uk) == h.U + 1 and uk[-1] == h.B and up[0] == 0
        multi = []
        for bm in range(h.NBR):
            k0, k1 = sp[bm], sp[bm + 1]
            slots = int(size[k0:k1].sum())
            u = max(1, -(-slots // unit_slots))
            assert up[bm + 1] - up[bm] == u
            assert np.all(us[up[bm]:up[bm + 1]] == bm)
            assert uk[up[bm]] == k0 and uk[up[bm + 1]] == k1          # units tile the stripe
            for i in range(u):
                k = uk[up[bm] + i]
                assert int(size[k0:k].sum()) * u >= i * slots          # the unit starts at its share ...
                assert k == k0 or int(size[k0:k - 1].sum()) * u < i * slots   # ... and not one entry later
                got = int(size[k:uk[up[bm] + i + 1]].sum())
                assert got <= slots / u + (size[k0:k1].max() if k1 > k0 else 0)
            if u > 1:
                multi.append(bm)
        assert np.array_equal(ms, np.array(multi, dtype=np.int32)) and h.NM == len(multi)
        if unit_slots == 64:
            assert h.NM > 0          # the case does split row blocks
        if unit_slots == 1 << 20:
            assert h.NM == 0 and h.U == h.NBR


def test_hash_groups_similar_rows(oracle):
    """Diagnostic of Section 4.1: the mean per-group standard deviation of row lengths does
    not grow when rows are put in hash order (it shrinks on varied inputs)."""
    m = make_config(5, scale=0.002)
    R, C, W = 512, 256, 32
    h = build(oracle, m, R=R, C=C, W=W)
    seg_len, row_local, slot_ptr = h.array("seg_len"), h.array("row_local"), h.array("slot_ptr")
    after, before = [], []
    for b in range(h.B):
        ln = seg_len[slot_ptr[b]:slot_ptr[b + 1]].astype(np.float64)
        if len(ln) < 2 * W:
            continue
        by_row = ln[np.argsort(row_local[slot_ptr[b]:slot_ptr[b + 1]], kind="stable")]
        for g0 in range(0, len(ln) - W + 1, W):
            after.append(ln[g0:g0 + W].std())
            before.append(by_row[g0:g0 + W].std())
    assert len(after) > 10 and np.mean(after) < np.mean(before)


def test_rejects_bad_parameters(oracle):
    m = worked_example_8x8()
    for kw in (dict(R=0), dict(C=0), dict(W=0), dict(R=70000), dict(C=70000), dict(num_workers=0)):
        with pytest.raises(ValueError):
            build(oracle, m, **{**dict(R=4, C=4, W=2), **kw})


@pytest.mark.parametrize("number,scale,R,C", [(1, 1.0, 512, 4096), (2, 0.002, 512, 4096), (3, 2**-8, 256, 1024),
                                              (4, 2**-9, 512, 2048), (5, 0.002, 512, 4096)])
def test_configs_small_scale(oracle, number, scale, R, C):
    m = make_config(number, scale)
    m.check()
    h = build(oracle, m, R=R, C=C, W=64)
    r, c, v = h.to_coo()
    order = np.lexsort((c, r))
    rows = np.repeat(np.arange(m.n_rows), np.diff(m.ptr))
    assert np.array_equal(r[order], rows) and np.array_equal(c[order], m.col)
    assert np.array_equal(v[order].view(np.uint32), m.val.view(np.uint32))
    y_ref, s = oracle.csr_spmv_f64(m.ptr, m.col, m.val, m.x)
    y, _ = h.spmv(m.x)
    assert np.all(np.abs(y - y_ref) <= 1e-12 * s)
    # per-row segment lengths add up to the row length
    tot = np.zeros(m.n_rows, dtype=np.int64)
    bm = np.repeat(h.array("blk_bm"), np.diff(h.array("slot_ptr")))
    np.add.at(tot, bm.astype(np.int64) * R + h.array("row_local"), h.array("seg_len"))
    assert np.array_equal(tot, np.diff(m.ptr))


def test_plain_2d_partition_keeps_row_order(oracle):
    """hash_shift = -2 (the plain 2D partitioning of Section 4): the slots of every block list its
    rows in ascending order, nothing else changes (same segments, same y)."""
    m = random_csr(200, 300, 0.08, 9)
    plain = build(oracle, m, R=32, C=64, W=8, hash_shift=-2)
    hbp = build(oracle, m, R=32, C=64, W=8)
    sp, rl = plain.array("slot_ptr"), plain.array("row_local")
    for b in range(plain.B):
        assert np.all(np.diff(rl[sp[b]:sp[b + 1]].astype(np.int64)) > 0)
    assert (plain.B, plain.S) == (hbp.B, hbp.S)
    assert coo_set(*plain.to_coo()) == coo_set(*hbp.to_coo())
    y_ref, s_abs = oracle.csr_spmv_f64(m.ptr, m.col, m.val, m.x)
    y, _ = plain.spmv(m.x)
    assert np.all(np.abs(y - y_ref) <= 1e-12 * np.maximum(s_abs, 1e-300))


def test_fp64_storage(oracle):
    """fp64 storage (Section 3.1's value type): the structure is that of the fp32 build of the same
    pattern, the values come back bit for bit (they are not float32-representable), and the SpMV
    agrees with the plain definition and with an exact rational evaluation on sampled rows."""
    from fractions import Fraction
    m32 = random_csr(150, 260, 0.07, 21, empty_row_frac=0.1)
    m = widen_to_f64(m32, 5)
    assert np.any(m.val != m.val.astype(np.float32)) and np.any(m.x != m.x.astype(np.float32))
    h32 = build(oracle, m32, R=32, C=64, W=8, num_workers=3)
    h = build(oracle, m, R=32, C=64, W=8, num_workers=3)
    for name in oracle.ARRAYS:
        if name != "data":
            assert np.array_equal(h.array(name), h32.array(name)), name
    assert h.array("data").dtype == np.float64 and h.array("data").shape == (m.nnz,)
    rows, cols, vals = h.to_coo()
    got = sorted(zip(rows.tolist(), cols.tolist(), vals.view(np.uint64).tolist()))
    want = sorted(zip(np.repeat(np.arange(m.n_rows), np.diff(m.ptr)).tolist(), m.col.tolist(), m.val.view(np.uint64).tolist()))
    assert got == want
    y_ref, s_abs = oracle.csr_spmv_f64(m.ptr, m.col, m.val, m.x)
    y, _ = h.spmv(m.x)
    assert np.all(np.abs(y - y_ref) <= 1e-13 * s_abs)
    for i in range(0, m.n_rows, 7):
        exact = sum((Fraction(float(m.val[j])) * Fraction(float(m.x[m.col[j]])) for j in range(m.ptr[i], m.ptr[i + 1])), Fraction(0))
        # the reference is the exact sum rounded: half an ulp of the result plus extended-precision noise
        assert abs(Fraction(float(y_ref[i])) - exact) <= Fraction(1, 2**53) * abs(exact) + Fraction(1, 2**60) * Fraction(float(s_abs[i]))
        assert abs(Fraction(float(y[i])) - exact) <= Fraction(1, 10**13) * Fraction(float(s_abs[i])) + Fraction(1, 10**300)
    # the float32 result of the same pattern differs by more than the fp64 bound on most rows
    y32, _ = oracle.csr_spmv_f64(m32.ptr, m32.col, m32.val, m32.x)
    assert np.mean(np.abs(y32 - y_ref) > 1e-11 * s_abs) > 0.5


def test_length_key_orders_rows_by_length(oracle):
    """hash_shift = -3 (the finest possible mapping of Section 5's outlook): the slots of every block
    are in ascending (length, row) order, which is what numpy's stable sort gives; nothing else changes."""
    m = random_csr(300, 400, 0.08, 17)
    by_len = build(oracle, m, R=64, C=128, W=8, hash_shift=-3)
    hbp = build(oracle, m, R=64, C=128, W=8)
    sp, rl, sl = by_len.array("slot_ptr"), by_len.array("row_local").astype(np.int64), by_len.array("seg_len").astype(np.int64)
    hsp, hrl, hsl = hbp.array("slot_ptr"), hbp.array("row_local").astype(np.int64), hbp.array("seg_len").astype(np.int64)
    assert np.array_equal(sp, hsp)
    for b in range(by_len.B):
        rows, lens = hrl[hsp[b]:hsp[b + 1]], hsl[hsp[b]:hsp[b + 1]]
        order = np.lexsort((rows, lens))                       # by length, then by row
        assert np.array_equal(rl[sp[b]:sp[b + 1]], rows[order])
        assert np.array_equal(sl[sp[b]:sp[b + 1]], lens[order])
    assert coo_set(*by_len.to_coo()) == coo_set(*hbp.to_coo())
    y_ref, s_abs = oracle.csr_spmv_f64(m.ptr, m.col, m.val, m.x)
    y, _ = by_len.spmv(m.x)
    assert np.all(np.abs(y - y_ref) <= 1e-12 * np.maximum(s_abs, 1e-300))


# ---------------------------------------------------------------- keys, per-block shift, the paper's schedule

def _hash_key_by_hand(n, a, R):
    """The hash of Section 3.2 written out again (aggregation, dispersion, linear mapping, clamp)."""
    b = max(1, R // 9)
    return min(min(n >> a, 8) * b + (((n % (1 << a)) * b) >> a), R - 1)


@pytest.mark.parametrize("mode", [-1, 2, -2, -3])
def test_slot_keys_are_the_keys_of_the_lengths(oracle, mode):
    """slot_key is what ordered the slots: the hash of the slot's own length with the matrix's shift
    (0 without reorder, the length itself in the length-key mode), non-decreasing inside a block."""
    m = make_config(5, 0.004)
    o = build(oracle, m, R=64, C=512, W=8, hash_shift=mode)
    key, n, sp = o.array("slot_key"), o.array("seg_len"), o.array("slot_ptr")
    want = (np.zeros_like(key) if mode == -2 else n.astype(np.uint32) if mode == -3
            else np.array([_hash_key_by_hand(int(v), o.a, 64) for v in n], dtype=np.uint32))
    assert np.array_equal(key, want)
    assert np.all(o.array("blk_shift") == o.a)
    for b in range(o.B):
        assert np.all(np.diff(key[sp[b]:sp[b + 1]].astype(np.int64)) >= 0)


def test_per_block_shift_by_brute_force(oracle):
    """hash_shift = -4: each block's shift is the smallest a with at least 15/16 of the block's own rows
    below 9 * 2^a (recounted here from the CSR arrays), its slots are in (key with that shift, row) order,
    and the nonzeros still round-trip."""
    m = make_config(4, 2**-9)   # R-MAT: dense and sparse blocks side by side
    R, C = 128, 256
    o = build(oracle, m, R=R, C=C, W=16, hash_shift=-4)
    rows = np.repeat(np.arange(m.n_rows), np.diff(m.ptr))
    bm, bn = rows // R, m.col // C
    shifts = o.array("blk_shift")
    assert len(set(shifts.tolist())) > 1, "the test matrix should need different shifts in different blocks"
    sp, rl, sl, key = o.array("slot_ptr"), o.array("row_local"), o.array("seg_len"), o.array("slot_key")
    for b in range(o.B):
        sel = (bm == o.array("blk_bm")[b]) & (bn == o.array("blk_bn")[b])
        lens = np.bincount(rows[sel] % R, minlength=R)
        lens_nz = lens[lens > 0]
        a = next((a for a in range(13) if 16 * np.count_nonzero(lens_nz < 9 * 2**a) >= 15 * len(lens_nz)), 12)
        assert shifts[b] == a
        order = sorted((_hash_key_by_hand(int(lens[r]), a, R), r) for r in np.flatnonzero(lens))
        assert [r for _, r in order] == rl[sp[b]:sp[b + 1]].tolist()
        assert [k for k, _ in order] == key[sp[b]:sp[b + 1]].tolist()
        assert [int(lens[r]) for _, r in order] == sl[sp[b]:sp[b + 1]].tolist()
    r2, c2, v2 = o.to_coo()
    assert coo_set(r2, c2, v2) == csr_coo(m)
    y, _ = o.spmv(m.x)
    y_ref, s_abs = oracle.csr_spmv_f64(m.ptr, m.col, m.val, m.x)
    assert np.all(np.abs(y - y_ref) <= 1e-12 * s_abs)


@pytest.mark.parametrize("P,q8", [(1, 256), (3, 224), (5, 100), (16, 256), (40, 0), (1000, 255)])
def test_paper_schedule_by_definition(oracle, P, q8):
    """Section 3.3 read literally: F = floor(B f / P) blocks per worker in list order (blocks of one
    column stay together: the list is column-major), the blocks from P F on behind one ticket counter;
    every block is walked exactly once."""
    m = random_csr(900, 1400, 0.02, 5, empty_row_frac=0.2)
    o = build(oracle, m, R=32, C=64, W=8, num_workers=P, fixed_q8=q8, paper_schedule=True)
    F = (o.B * q8) // (256 * P)
    assert o.first_ticket_block == P * F and P * F <= o.B
    bgp, fs = o.array("blk_group_ptr"), o.array("fixed_start")
    assert fs.tolist() == [int(bgp[w * F]) for w in range(P + 1)]
    assert np.array_equal(o.array("comp_lo"), fs[1:])          # nothing inside a range is competitive
    covered = []
    for w in range(P):
        covered += list(range(w * F, (w + 1) * F))
        if F:
            assert o.array("fixed_col")[w] == o.array("blk_bn")[w * F]
            assert o.array("comp_col")[w] == o.array("blk_bn")[(w + 1) * F - 1]
    covered += list(range(P * F, o.B))                          # claimed one by one
    assert covered == list(range(o.B))
    # the layout itself does not depend on the schedule
    o0 = build(oracle, m, R=32, C=64, W=8, num_workers=P, fixed_q8=q8)
    for name in ("row_local", "seg_len", "col_local", "data", "group_ptr", "slot_key"):
        assert np.array_equal(o.array(name), o0.array(name))
    assert o0.first_ticket_block == -1
