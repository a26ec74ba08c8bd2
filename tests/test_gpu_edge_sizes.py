"""Edges of the supported range: the largest W one linear may have (byte offsets just below 2^31), the longest
lists (LSW_MAX_K old + LSW_MAX_K new experts), and the smallest everything."""
import numpy as np
import pytest
import torch

from oracle import lsw_oracle as O
from paper_2405_17741_amd import binding as L
from paper_2405_17741_amd import inputs as I
from tests.gpu_harness import DeviceStack, check_step, gate_quality, merge_reports

pytestmark = pytest.mark.gpu
NONE = (np.zeros(0, np.int32), np.zeros(0, np.float32))


@pytest.mark.parametrize("kernel", [L.KERNEL_VALU, L.KERNEL_MFMA])
def test_largest_single_weight(kernel):
    """16384 x 65528 bf16 = 2^31 - 262144 bytes: the last rows' byte offsets need all 31 bits."""
    out, inn, E, r = 16384, 65528, 2, 8
    assert out * inn * 2 < 2 ** 31 <= (out + 128) * inn * 2
    g = torch.Generator(device="cuda"); g.manual_seed(99)
    W = (torch.randn(out, inn, generator=g, device="cuda") * 0.02).to(torch.bfloat16)
    A = torch.randn(E, r, inn, generator=g, device="cuda") / 256
    B = torch.randn(E, out, r, generator=g, device="cuda") * 0.01
    ds = DeviceStack([(W, A, B)], [(0, 0, out, inn)], E, r, kernel=kernel)
    rows = np.array([0, 1, 127, 128, 8191, 8192, 16255, 16256, 16382, 16383], dtype=np.int64)
    A_h = A.cpu().numpy()
    B_h = B.index_select(1, torch.as_tensor(rows, device="cuda")).cpu().numpy()
    steps = [NONE, (np.array([1], np.int32), np.array([1.0], np.float32)),
             (np.array([0, 1], np.int32), np.array([0.3, 0.7], np.float32)), NONE]
    reports = []
    for old, new in zip(steps[:-1], steps[1:]):
        before = ds.rows(0, rows)
        guard = W[-1, -8:].clone()
        ds.switch(old, new)
        got = ds.rows(0, rows)
        rep, _ = check_step(before, got, A_h, B_h, old, new)
        assert rep["fail"] == 0, {k: v for k, v in rep.items() if k != "fail_mask"}
        assert not torch.equal(W[-1, -8:], guard)          # the very last 16 bytes were updated
        reports.append(rep)
    gate_quality(merge_reports(reports), "largest single weight", exact_min=0.9998, clause2_max=2e-5)
    ds.close()
    # one more row of 128 would cross 2^31 bytes: refused at create time, before any launch
    with pytest.raises(L.LswError) as e:
        L.lsw_create_adapters([(W.data_ptr(), A.data_ptr(), B.data_ptr(), out + 1, inn, 0, 0)], E, r)
    assert e.value.status == L.LSW_ERR_SHAPE


def test_longest_lists_and_smallest_shapes():
    rng = np.random.default_rng(77)
    # 8 old + 8 new distinct experts of rank 8: 16 terms, fused rank 128 (chunked matrix-core kernel)
    out, inn, E, r = 200, 520, 16, 8
    W, A, B = I.host_linear(rng, out, inn, E, r, 0.02, 1 / 16, 0.01)
    for kernel in (L.KERNEL_VALU, L.KERNEL_MFMA):
        ds = DeviceStack.from_host([(W, A, B)], [(0, 0, out, inn)], E, r, kernel=kernel)
        perm = rng.permutation(E).astype(np.int32)
        g = rng.random(E).astype(np.float32)
        old = (perm[:8].copy(), (g[:8] / g[:8].sum()).astype(np.float32))
        new = (perm[8:].copy(), (g[8:] / g[8:].sum()).astype(np.float32))
        mixed = (np.concatenate([perm[4:8], perm[8:12]]).astype(np.int32), np.full(8, 0.125, np.float32))   # 4 shared with each
        prev = ds.rows(0)
        for a, b in [(NONE, old), (old, new), (new, mixed), (mixed, NONE)]:
            ds.switch(a, b)
            assert L.lsw_query(ds.ctx, L.LSW_Q_LAST_KERNEL) == kernel
            got = ds.rows(0)
            rep, _ = check_step(prev, got, A, B, a, b)
            assert rep["fail"] == 0, (kernel, {k: v for k, v in rep.items() if k != "fail_mask"})
            prev = got
        with pytest.raises(L.LswError):
            ds.switch(NONE, (np.arange(9, dtype=np.int32), np.full(9, 1 / 9, np.float32)))      # k > LSW_MAX_K
        ds.close()
    # one expert, one row, eight columns
    W, A, B = I.host_linear(rng, 1, 8, 1, 8, 0.02, 0.5, 0.1)
    for kernel in (L.KERNEL_VALU, L.KERNEL_MFMA):
        ds = DeviceStack.from_host([(W, A, B)], [(0, 0, 1, 8)], 1, 8, kernel=kernel)
        one = (np.array([0], np.int32), np.array([1.0], np.float32))
        prev = ds.rows(0)
        for a, b in [(NONE, one), (one, NONE)]:
            ds.switch(a, b)
            got = ds.rows(0)
            rep, _ = check_step(prev, got, A, B, a, b)
            assert rep["fail"] == 0
            prev = got
        ds.close()


def test_many_distinct_layer_subsets_meet_a_limit_not_an_eviction():
    """Every new layer subset gets a small device table that is never moved or freed while the context lives (launches
    in flight and recorded graphs hold its address); a context keeps at most 256 of them.  600 different subsets of a
    10-layer stack, each merged and unmerged: beyond the limit the call fails with LSW_ERR_STATE and touches nothing,
    lsw_drop_subset_tables frees the tables, the owned bytes stay bounded and the weights stay right."""
    E, r, layers = 4, 8, 10
    rng = np.random.default_rng(31)
    host = [I.host_linear(rng, 64, 256, E, r, 0.02, 1 / 16, 0.01) for _ in range(layers)]
    shapes = [(l, 0, 64, 256) for l in range(layers)]
    ds = DeviceStack.from_host(host, shapes, E, r, kernel=L.KERNEL_MFMA)
    base_bytes = L.lsw_query(ds.ctx, L.LSW_Q_PACKED_BYTES)
    a = (np.array([1, 3], np.int32), np.array([0.25, 0.75], np.float32))
    peak, refused = 0, 0
    for mask in range(1, 601):
        subset = [l for l in range(layers) if (mask >> l) & 1]
        checked = mask % 97 == 0                             # now and then: the subset, and only it, was merged
        if checked:
            prev = [ds.rows(p) for p in range(layers)]
        try:
            ds.switch(NONE, a, layers=subset)
        except L.LswError as e:
            assert e.status == L.LSW_ERR_STATE and "lsw_drop_subset_tables" in str(e)
            refused += 1
            L.lsw_drop_subset_tables(ds.ctx)
            assert L.lsw_query(ds.ctx, L.LSW_Q_PACKED_BYTES) == base_bytes
            ds.switch(NONE, a, layers=subset)
        if checked:
            for p in range(layers):
                got = ds.rows(p)
                if p in subset:
                    rep, _ = check_step(prev[p], got, host[p][1], host[p][2], NONE, a)
                    assert rep["fail"] == 0
                else:
                    assert (got == prev[p]).all()
        ds.switch(a, NONE, layers=subset)
        peak = max(peak, L.lsw_query(ds.ctx, L.LSW_Q_PACKED_BYTES))
    assert refused == 2                                      # 600 subsets, 256 tables at a time
    assert peak - base_bytes <= 257 * (2 * layers + 1) * 4
    # merge and unmerge are not exact inverses in bf16 (one rounding each), so the state now is whatever 600 such pairs
    # left; one more switch from it is checked like any other
    before = [ds.rows(p) for p in range(layers)]
    ds.switch(NONE, a)
    for p in range(layers):
        rep, _ = check_step(before[p], ds.rows(p), host[p][1], host[p][2], NONE, a)
        assert rep["fail"] == 0
    ds.close()


def test_options_reject_values_outside_their_documented_range():
    rng = np.random.default_rng(3)
    host = [I.host_linear(rng, 32, 64, 2, 8, 0.02, 1 / 8, 0.01)]
    ds = DeviceStack.from_host(host, [(0, 0, 32, 64)], 2, 8)
    bad = [(L.LSW_OPT_KERNEL, 3), (L.LSW_OPT_GRID, -1), (L.LSW_OPT_TILE_COLS, 100), (L.LSW_OPT_TILE_COLS, 0),
           (L.LSW_OPT_XCD_REMAP, 4), (L.LSW_OPT_XCD_REMAP, -1), (L.LSW_OPT_PANEL_GROUP, -2), (L.LSW_OPT_PANEL_GROUP, 2000),
           (L.LSW_OPT_XCD_POOL, -1), (L.LSW_OPT_GEMV_GRID, -5), (99, 0)]
    for opt, value in bad:
        with pytest.raises(L.LswError) as e:
            L.lsw_set_option(ds.ctx, opt, value)
        assert e.value.status == L.LSW_ERR_ARG, (opt, value)
    for opt, value in [(L.LSW_OPT_XCD_REMAP, 0), (L.LSW_OPT_XCD_REMAP, 3), (L.LSW_OPT_PANEL_GROUP, -1), (L.LSW_OPT_PANEL_GROUP, 4),
                       (L.LSW_OPT_XCD_POOL, 0), (L.LSW_OPT_XCD_POOL, 32), (L.LSW_OPT_TILE_COLS, 512)]:
        L.lsw_set_option(ds.ctx, opt, value)
    assert L.lsw_query(ds.ctx, 99) == -1
    # the stack still switches correctly under those settings
    a = (np.array([1], np.int32), np.array([1.0], np.float32))
    before = ds.rows(0)
    ds.switch(NONE, a)
    rep, _ = check_step(before, ds.rows(0), host[0][1], host[0][2], NONE, a)
    assert rep["fail"] == 0
    ds.close()
