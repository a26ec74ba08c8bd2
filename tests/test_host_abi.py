"""CPU-side checks of the C-ABI library: it loads, exports what include/lsw.h declares, and its
host logic (router, term list, work decomposition, argument validation) behaves as documented.
No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import lsw_oracle as O
from paper_2405_17741_amd import binding as L
from paper_2405_17741_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("lsw.h", "lsw_tuning.h"))
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(lsw_[a-z0-9_]+)\s*\(", header))
    assert declared == set(L.EXPORTS)
    lib = L.lib()
    for name in declared:
        assert getattr(lib, name) is not None


def test_route_matches_oracle_bit_for_bit_on_ids():
    rng = np.random.default_rng(0)
    worst = 0
    for E, k in [(8, 2), (16, 2), (8, 1), (16, 4), (8, 8), (3, 0)]:
        for _ in range(300):
            l = rng.normal(0, 1, E).astype(np.float32)
            if rng.random() < 0.3:                      # plant ties
                l[rng.integers(0, E)] = l[rng.integers(0, E)]
            ids, gates = L.lsw_route(l, k)
            oids, ogates = O.route(l, k)
            assert ids.tolist() == oids.tolist()
            if k:
                d = np.abs(gates.view(np.int32).astype(np.int64) - ogates.view(np.int32).astype(np.int64)).max()
                worst = max(worst, int(d))
    assert worst <= 1          # gates within one fp32 ulp of the oracle's


def test_route_crafted_ties_and_errors():
    assert L.lsw_route(np.array([1, 1, 0, 1], np.float32), 2)[0].tolist() == [0, 1]
    assert L.lsw_route(np.array([-0.0, 0.0, -1.0], np.float32), 2)[0].tolist() == [0, 1]
    ids, gates = L.lsw_route(np.zeros(8, np.float32), 2)
    assert ids.tolist() == [0, 1] and gates.tolist() == [0.5, 0.5]
    ids, gates = L.lsw_route(np.array([3.0, 7.0], np.float32), 1)
    assert ids.tolist() == [1] and gates.tolist() == [1.0]
    for bad in [lambda: L.lsw_route(np.array([0.0, np.nan], np.float32), 1),
                lambda: L.lsw_route(np.zeros(4, np.float32), 5),
                lambda: L.lsw_route(np.zeros(4, np.float32), -1)]:
        with pytest.raises(L.LswError) as e:
            bad()
        assert e.value.status == L.LSW_ERR_ARG
    assert "NaN" in L.lsw_last_error() or "k=" in L.lsw_last_error()


def _dense_terms(ids, coeff, E):
    v = np.zeros(E, np.float64)
    for e, c in zip(ids.tolist(), coeff.tolist()):
        assert v[e] == 0.0, "an expert appears twice in the term list"
        v[e] = c
    return v


def test_build_terms_equals_signed_gate_vector():
    rng = np.random.default_rng(1)
    for _ in range(500):
        E = int(rng.integers(2, 17))
        ko, kn = int(rng.integers(0, min(E, 4) + 1)), int(rng.integers(0, min(E, 4) + 1))
        oi = rng.choice(E, ko, replace=False).astype(np.int32)
        ni = rng.choice(E, kn, replace=False).astype(np.int32)
        og = rng.random(ko).astype(np.float32)
        ng = rng.random(kn).astype(np.float32)
        scale = float(rng.choice([1.0, 0.25, 2.0]))
        ids, coeff = L.lsw_build_terms(oi, og, ni, ng, E, scale)
        want = np.zeros(E, np.float64)
        for e, g in zip(ni.tolist(), ng.tolist()):
            want[e] += scale * float(g)
        for e, g in zip(oi.tolist(), og.tolist()):
            want[e] -= scale * float(g)
        got = _dense_terms(ids, coeff, E)
        assert np.allclose(got, want, rtol=0, atol=2.0 ** -23 * scale)
        assert (coeff != 0).all()
        assert len(ids) <= ko + kn


def test_build_terms_cancels_identical_pairs_and_orders_new_first():
    ids, coeff = L.lsw_build_terms([2, 5], [0.6, 0.4], [5, 2], [0.4, 0.6], 8)
    assert len(ids) == 0
    ids, coeff = L.lsw_build_terms([2, 5], [0.6, 0.4], [5, 7], [0.5, 0.5], 8)
    assert ids.tolist() == [5, 7, 2]
    assert coeff.tolist() == [np.float32(0.5) - np.float32(0.4), 0.5, -np.float32(0.6)]
    ids, coeff = L.lsw_build_terms([], [], [1], [1.0], 8, 0.25)
    assert ids.tolist() == [1] and coeff.tolist() == [0.25]
    ids, coeff = L.lsw_build_terms([1], [1.0], [], [], 8)
    assert ids.tolist() == [1] and coeff.tolist() == [-1.0]


@pytest.mark.parametrize("args", [
    dict(old_ids=[0, 0], old_gates=[0.5, 0.5], new_ids=[], new_gates=[]),            # duplicate id
    dict(old_ids=[], old_gates=[], new_ids=[8], new_gates=[1.0]),                    # id out of range
    dict(old_ids=[-1], old_gates=[1.0], new_ids=[], new_gates=[]),
    dict(old_ids=[], old_gates=[], new_ids=[1], new_gates=[float("nan")]),           # non-finite gate
    dict(old_ids=[], old_gates=[], new_ids=[1], new_gates=[float("inf")]),
    dict(old_ids=list(range(9)), old_gates=[0.1] * 9, new_ids=[], new_gates=[]),     # k > LSW_MAX_K
])
def test_build_terms_rejects_bad_lists(args):
    with pytest.raises(L.LswError) as e:
        L.lsw_build_terms(args["old_ids"], args["old_gates"], args["new_ids"], args["new_gates"], 8 if len(args["old_ids"]) < 9 else 16)
    assert e.value.status == L.LSW_ERR_ARG


@pytest.mark.parametrize("tile", [(64, 128), (32, 1024), (7, 24)])
def test_worklist_partitions_every_weight_exactly_once(tile):
    tr, tc = tile
    out = np.array([256, 100, 33, 64, 1], np.int32)
    inn = np.array([256, 1048, 8, 2000, 136], np.int32)
    n = L.lsw_worklist_size(out, inn, tr, tc)
    assert n == sum(-(-int(o) // tr) * -(-int(i) // tc) for o, i in zip(out, inn))
    cover = [np.zeros((o, i), np.int32) for o, i in zip(out, inn)]
    last = (-1, -1, -1)
    for it in range(n):
        lin, r0, nr, c0, nc = L.lsw_worklist_item(out, inn, tr, tc, it)
        assert 0 < nr <= tr and 0 < nc <= tc and r0 % tr == 0 and c0 % tc == 0
        cover[lin][r0:r0 + nr, c0:c0 + nc] += 1
        assert (lin, r0, c0) > last           # linear by linear, rows outermost
        last = (lin, r0, c0)
    for c in cover:
        assert (c == 1).all()
    with pytest.raises(L.LswError):
        L.lsw_worklist_item(out, inn, tr, tc, n)
    assert L.lsw_worklist_size(out, inn, 0, tc) == -1


@pytest.mark.parametrize("group", [1, 2, 3, 4, 8])
def test_grouped_worklist_is_a_permutation_of_the_plain_one(group):
    """Panels in groups: inside a linear with more panels than the group size, all row blocks of one group of panels come
    before the next group; the set of tiles is the same as in the plain order, each exactly once."""
    tr, tc = 32, 256
    out = np.array([256, 100, 33, 64, 1, 96], np.int32)
    inn = np.array([256, 1048, 8, 2000, 136, 2816], np.int32)      # 1, 5, 1, 8, 1, 11 panels
    n = L.lsw_worklist_size(out, inn, tr, tc)
    plain = {L.lsw_worklist_item(out, inn, tr, tc, it) for it in range(n)}
    seen = []
    for it in range(n):
        seen.append(L.lsw_worklist_item_grouped(out, inn, tr, tc, group, it))
    assert len(set(seen)) == n and set(seen) == plain
    assert [s[0] for s in seen] == sorted(s[0] for s in seen)                       # still linear by linear
    for lin in range(len(out)):
        mine = [s for s in seen if s[0] == lin]
        panels = -(-int(inn[lin]) // tc)
        if panels <= group:                                                           # few panels: the plain order
            assert mine == sorted(mine, key=lambda s: (s[1], s[3]))
        else:                                                                         # group of the panel never decreases; rows outermost inside
            keys = [(s[3] // tc // group, s[1], s[3]) for s in mine]
            assert keys == sorted(keys)
    assert L.lsw_worklist_item_grouped(out, inn, tr, tc, 0, 7) == L.lsw_worklist_item(out, inn, tr, tc, 7)
    with pytest.raises(L.LswError):
        L.lsw_worklist_item_grouped(out, inn, tr, tc, -1, 0)


@pytest.mark.parametrize("n_items,grid,pool_div", [(49408, 256, 16), (49408, 256, 0), (1299, 64, 16), (614, 64, 16), (141, 64, 16),
                                                  (5, 256, 16), (0, 8, 16), (4096, 256, 3), (12345, 248, 16), (263, 16, 2)])
def test_per_xcd_walk_hands_out_every_item_exactly_once(n_items, grid, pool_div):
    """Static columns of all workgroups plus the pool claims cover [0, n_items) exactly once; with a pool every workgroup
    keeps at least two static items; claims beyond the pool stand for nothing."""
    taken = np.zeros(n_items, np.int32)
    pool_len = None
    for block in range(grid):
        first, step, static_end, per, pl = L.lsw_walk_share(n_items, grid, block, pool_div)
        assert step == grid // 8 and per == -(-n_items // 8)
        pool_len = pl if pool_len is None else pool_len
        assert pl == pool_len                                  # the same decision in every workgroup
        mine = list(range(first, static_end, step))
        if pl > 0:
            assert len(mine) >= 2
        for it in mine:
            taken[it] += 1
    if pool_div <= 0:
        assert pool_len == 0
    for g in range(8 * pool_len):
        it = L.lsw_walk_pool_item(n_items, grid, pool_div, g)
        assert 0 <= it < n_items
        taken[it] += 1
    assert (taken == 1).all()
    for g in (8 * pool_len, 8 * pool_len + 1, 8 * pool_len + 255, -1):
        assert L.lsw_walk_pool_item(n_items, grid, pool_div, g) == -1
    with pytest.raises(L.LswError):
        L.lsw_walk_share(n_items, grid + 1, 0, pool_div)
    with pytest.raises(L.LswError):
        L.lsw_walk_share(n_items, grid, grid, pool_div)


def test_worklist_counts_of_the_7b_workload():
    shapes = I.WORKLOADS["7b"].linear_shapes()
    out = np.array([s[2] for s in shapes], np.int32)
    inn = np.array([s[3] for s in shapes], np.int32)
    # 128x128 tiles: the count quoted for the 7B-shaped stack
    assert L.lsw_worklist_size(out, inn, 128, 128) == 395_264
    assert L.lsw_worklist_size(out, inn, 32, 1024) == 32 * (4 * 128 * 4 + 2 * 344 * 4 + 128 * 11)


def _fake_linear(out=64, inn=64, w=0x1000, a=0x2000, b=0x3000, layer=0):
    return (w, a, b, out, inn, layer, 0)


@pytest.mark.parametrize("lin,E,r,scale,status", [
    ([], 8, 8, 1.0, L.LSW_ERR_ARG),
    ([_fake_linear()], 0, 8, 1.0, L.LSW_ERR_ARG),
    ([_fake_linear()], 8, 0, 1.0, L.LSW_ERR_ARG),
    ([_fake_linear()], 8, 8, float("nan"), L.LSW_ERR_ARG),
    ([_fake_linear(w=0)], 8, 8, 1.0, L.LSW_ERR_ARG),
    ([_fake_linear(layer=-1)], 8, 8, 1.0, L.LSW_ERR_ARG),
    ([_fake_linear(out=0)], 8, 8, 1.0, L.LSW_ERR_SHAPE),
    ([_fake_linear(inn=12)], 8, 8, 1.0, L.LSW_ERR_SHAPE),
    ([_fake_linear(inn=0)], 8, 8, 1.0, L.LSW_ERR_SHAPE),
    ([_fake_linear(w=0x1008)], 8, 8, 1.0, L.LSW_ERR_SHAPE),
    ([_fake_linear(a=0x2004)], 8, 8, 1.0, L.LSW_ERR_SHAPE),
])
def test_create_validates_before_touching_any_device(lin, E, r, scale, status):
    with pytest.raises(L.LswError) as e:
        L.lsw_create_adapters(lin, E, r, scale)
    assert e.value.status == status
    assert L.lsw_last_error()


@pytest.mark.parametrize("r,dtype,status", [
    (4, L.LSW_FACTOR_BF16, L.LSW_ERR_SHAPE),      # bf16 rows of B must stay 16-byte aligned
    (8, 2, L.LSW_ERR_ARG),                        # unknown storage type
    (8, -1, L.LSW_ERR_ARG),
])
def test_create_ex_validates_the_factor_dtype(r, dtype, status):
    with pytest.raises(L.LswError) as e:
        L.lsw_create_adapters([_fake_linear()], 8, r, 1.0, dtype)
    assert e.value.status == status


def test_null_context_calls_fail_cleanly():
    lib = L.lib()
    assert lib.lsw_switch(None, None, 0, None, None, 0, None, None, 0, None) == L.LSW_ERR_ARG
    assert lib.lsw_merged_gemv(None, 0, None, None, None) == L.LSW_ERR_ARG
    assert lib.lsw_set_option(None, 1, 0) == L.LSW_ERR_ARG
    assert lib.lsw_query(None, 1) == -1
    k = ctypes.c_int32(0)
    assert lib.lsw_get_state(None, 0, None, None, ctypes.byref(k)) == L.LSW_ERR_ARG
    lib.lsw_destroy(None)


@pytest.mark.parametrize("rows,cols,grid", [
    ((2048,) * 7, (4096, 4096, 4096, 4096, 11008, 11008, 4096), 256),       # the 7B layer at 2048 tokens
    ((1,), (8,), 256),                                                       # one unit: 255 empty ranges
    ((300, 300, 300), (264, 520, 136), 64), ((37,), (11000,), 8), ((129, 1), (256, 257), 16), ((130,) * 8, (72,) * 8, 256),
])
def test_flat_order_of_the_prompt_path_covers_every_cell_once_in_equal_ranges(rows, cols, grid):
    """The up-projection of the prompt path: every workgroup's items together cover every cell of every output exactly
    once, an item never leaves its row block or its matrix, its columns start and end on 256-column steps (or at the edge),
    and no workgroup has more than one unit (128 rows x 256 columns) more than another."""
    cover = [np.zeros(((r + 127) // 128, (c + 255) // 256), np.int32) for r, c in zip(rows, cols)]
    per_block = []
    for block in range(grid):
        units, unit = 0, -1
        while True:
            mat, row0, col0, n_cols, nxt = L.lsw_flat_item(rows, cols, grid, block, unit)
            if mat < 0:
                assert unit == -1 and nxt == -1                # an empty range says so at once
                break
            assert 0 <= mat < len(rows) and row0 % 128 == 0 and row0 < rows[mat] and col0 % 256 == 0 and n_cols > 0
            assert col0 + n_cols <= cols[mat] and ((col0 + n_cols) % 256 == 0 or col0 + n_cols == cols[mat])
            n = (n_cols + 255) // 256
            cover[mat][row0 // 128, col0 // 256: col0 // 256 + n] += 1
            units += n
            if nxt < 0:
                break
            unit = nxt
        per_block.append(units)
    assert all((c == 1).all() for c in cover)
    assert max(per_block) - min(per_block) <= 1
    # each XCD (blocks x, x + 8, ...) works on one contiguous eighth: its blocks' first units rise with the block number
    firsts = {}
    for block in range(grid):
        mat, row0, col0, _, _ = L.lsw_flat_item(rows, cols, grid, block)
        if mat >= 0:
            firsts.setdefault(block % 8, []).append((mat, row0, col0))
    assert all(v == sorted(v) for v in firsts.values())
    with pytest.raises(L.LswError):
        L.lsw_flat_item(rows, cols, grid + 1, 0)
    with pytest.raises(L.LswError):
        L.lsw_flat_item(rows, cols, grid, grid)

