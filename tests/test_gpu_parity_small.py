"""GPU parity of lsw_switch against the CPU oracle on small workloads (full matrices, every step).

Bar: every element within 1 bf16 ulp of the oracle applied to the GPU's own previous state (or within
one bf16 ulp at the largest magnitude entering the sum, for results that cancel towards zero -- see
oracle/compare.py); hand-derived rounding fixtures bit-exact; invariants bit-exact."""
import numpy as np
import pytest
import torch

from oracle import lsw_oracle as O
from paper_2405_17741_amd import binding as L
from paper_2405_17741_amd import inputs as I
from tests.golden_cases import load_rne_cases
from tests.gpu_harness import bf16_factor_stack, DeviceStack, bits_to_device, check_step, device_to_bits, gate_quality, merge_reports

pytestmark = pytest.mark.gpu
KERNELS = [L.KERNEL_VALU, L.KERNEL_MFMA]
# Quality gates of the small workloads (see gpu_harness.gate_quality).  Their updates are 4 times larger against the
# weights than those of the model-shaped stacks (A has standard deviation 1/16), so more elements sit near a rounding
# boundary: measured 0.99996-0.999995 bit-equal and at most 2.5e-6 on the second clause with fp32 accumulation (the
# vector-ALU kernel), 0.99934-0.99981 and at most 5.3e-5 with the three-pass split on the matrix cores.
SMALL_GATES = {L.KERNEL_VALU: dict(exact_min=0.9999, clause2_max=1e-5), L.KERNEL_MFMA: dict(exact_min=0.999, clause2_max=1.5e-4)}


def _route_stream(wl, steps):
    logits = I.router_logits(wl, steps)
    return [O.route(l, wl.top_k) for l in logits]


@pytest.mark.parametrize("kernel", KERNELS)
def test_tiny_workload_every_step_full_matrix(kernel):
    wl = I.WORKLOADS["tiny"]
    host = I.host_stack(wl)
    ds = DeviceStack.from_host(host, wl.linear_shapes(), wl.experts, wl.rank, kernel=kernel)
    (W0, A, B), = host
    routes = _route_stream(wl, wl.steps)
    old = (np.zeros(0, np.int32), np.zeros(0, np.float32))
    prev = ds.rows(0)
    assert (prev == W0).all()
    free = W0.copy()
    reports = []
    for t, new in enumerate(routes):
        ds.switch(old, new)
        assert L.lsw_query(ds.ctx, L.LSW_Q_LAST_KERNEL) == kernel
        got = ds.rows(0)
        rep, want = check_step(prev, got, A, B, old, new)
        assert rep["fail"] == 0, (t, {k: v for k, v in rep.items() if k != "fail_mask"})
        reports.append(rep)
        free = O.switch_step(free, A, B, old[0], old[1], new[0], new[1])
        prev, old = got, new
    tot = merge_reports(reports)
    print(f"\n[tiny kernel={kernel}] {tot}; free-running mismatch after {wl.steps} steps: "
          f"{(free != prev).mean():.4%}")
    gate_quality(tot, f"tiny kernel={kernel}", **SMALL_GATES[kernel])
    # restore the base weights: within the drift the oracle itself predicts
    ds.switch(old, (np.zeros(0, np.int32), np.zeros(0, np.float32)))
    rep, _ = check_step(prev, ds.rows(0), A, B, old, (np.zeros(0, np.int32), np.zeros(0, np.float32)))
    assert rep["fail"] == 0
    ds.close()


@pytest.mark.parametrize("kernel", KERNELS)
def test_hand_derived_rounding_cases_bit_exact(kernel):
    cases = load_rne_cases()
    r = 8 if kernel != L.KERNEL_VALU else 1
    n = len(cases)
    # one linear per case: W is 1x8 with the case in column 3; only rank 0 of expert 0 is non-zero
    host, shapes = [], []
    for i, c in enumerate(cases):
        W = np.full((1, 8), 0x3F80, np.uint16)
        W[0, 3] = c["w"]
        A = np.zeros((1, r, 8), np.float32)
        B = np.zeros((1, 1, r), np.float32)
        A[0, 0, 3] = c["a"]
        B[0, 0, 0] = c["b"]
        host.append((W, A, B))
        shapes.append((i, 0, 1, 8))
    ds = DeviceStack.from_host(host, shapes, 1, r, kernel=kernel)
    for i, c in enumerate(cases):
        g = np.array([c["gate"]], np.float32)
        e = np.zeros(1, np.int32)
        none = (np.zeros(0, np.int32), np.zeros(0, np.float32))
        if c["side"] == "new":
            ds.switch(none, (e, g), layers=[i])
        else:
            ds.switch((e, g), none, layers=[i])
    bad = []
    for i, c in enumerate(cases):
        got = ds.rows(i)
        assert (np.delete(got[0], 3) == 0x3F80).all(), "neighbouring elements must not change"
        if c["tag"] == "":
            if int(got[0, 3]) != c["expect"]:
                bad.append((i, c, hex(int(got[0, 3]))))
        else:   # fp64-only ties and subnormal products: one ulp allowed
            from oracle.compare import ulp_distance
            assert ulp_distance(got[0, 3], np.uint16(c["expect"])) <= 1, (c, hex(int(got[0, 3])))
            print(f"[tagged {c['tag']}] expect {c['expect']:#06x} got {int(got[0,3]):#06x}")
    assert not bad, bad
    ds.close()


SHAPES = [
    # out, in, E, r
    (37, 8, 5, 8), (100, 264, 5, 8), (64, 1048, 4, 16), (33, 2056, 3, 8), (130, 520, 6, 24), (1, 16, 2, 8),
    (96, 256, 8, 32), (65, 136, 3, 4), (40, 72, 4, 1), (70, 1032, 4, 3),
    # fused ranks above 64: the chunked matrix-core kernel (2, 3 and 4 chunks per step), ragged rows and columns
    (150, 776, 5, 64), (129, 264, 4, 32), (33, 4360, 4, 48), (260, 520, 6, 40),
]


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("shape", SHAPES)
def test_ragged_shapes_and_term_counts(shape, kernel):
    out, inn, E, r = shape
    if kernel != L.KERNEL_VALU and r % 8:
        pytest.skip("matrix-core kernel needs r % 8 == 0")
    rng = np.random.default_rng(out * 1000 + inn + r)
    W, A, B = I.host_linear(rng, out, inn, E, r, 0.02, 1 / 16, 0.01)
    ds = DeviceStack.from_host([(W, A, B)], [(0, 0, out, inn)], E, r, scale=0.5, kernel=L.KERNEL_AUTO)
    none = (np.zeros(0, np.int32), np.zeros(0, np.float32))
    seq = [none]
    kmax = min(E, 2 if r > 16 else 3)
    kernels_used = set()
    for _ in range(6):
        k = int(rng.integers(1, kmax + 1))
        ids = rng.choice(E, k, replace=False).astype(np.int32)
        g = rng.random(k).astype(np.float32)
        seq.append((ids, (g / g.sum()).astype(np.float32)))
    seq.append(none)
    prev = ds.rows(0)
    reports = []
    for old, new in zip(seq[:-1], seq[1:]):
        n_terms = len(L.lsw_build_terms(old[0], old[1], new[0], new[1], E, 0.5)[0])
        fits = r % 8 == 0 and n_terms * (r // 8) <= 32
        use = kernel if (kernel == L.KERNEL_VALU or fits) else L.KERNEL_VALU
        L.lsw_set_option(ds.ctx, L.LSW_OPT_KERNEL, use)
        ds.switch(old, new)
        kernels_used.add(L.lsw_query(ds.ctx, L.LSW_Q_LAST_KERNEL))
        got = ds.rows(0)
        rep, _ = check_step(prev, got, A, B, old, new, scale=0.5)
        assert rep["fail"] == 0, (old, new, {k: v for k, v in rep.items() if k != "fail_mask"})
        reports.append(rep)
        prev = got
    gate_quality(merge_reports(reports), f"ragged {shape} kernel={kernel}", **SMALL_GATES[kernel])
    if kernel == L.KERNEL_MFMA and r >= 32:
        assert L.KERNEL_MFMA in kernels_used
    ds.close()


@pytest.mark.parametrize("shape", [(100, 264, 5, 8), (130, 1048, 6, 8), (33, 2056, 3, 8), (260, 4104, 4, 8)])
def test_streaming_matrix_core_kernel_with_the_resident_one_switched_off(shape):
    """Fused ranks up to 32 with fp32 factors normally run the resident-A kernel; LSW_OPT_RESIDENT_Q = 0 sends the same
    launches to the kernel that streams A per step.  Both must meet the bar, and they compute the same sums in the same
    order: bit-identical results."""
    out, inn, E, r = shape
    rng = np.random.default_rng(out * 31 + inn)
    W, A, B = I.host_linear(rng, out, inn, E, r, 0.02, 1 / 16, 0.01)
    a = DeviceStack.from_host([(W, A, B)], [(0, 0, out, inn)], E, r, kernel=L.KERNEL_MFMA)
    b = DeviceStack.from_host([(W, A, B)], [(0, 0, out, inn)], E, r, kernel=L.KERNEL_MFMA)
    L.lsw_set_option(b.ctx, L.LSW_OPT_RESIDENT_Q, 0)
    none = (np.zeros(0, np.int32), np.zeros(0, np.float32))
    seq = [none, (np.array([1, 2], np.int32), np.array([0.7, 0.3], np.float32)),
           (np.array([2, 0], np.int32), np.array([0.45, 0.55], np.float32)), (np.array([1], np.int32), np.array([1.0], np.float32)), none]
    prev = a.rows(0)
    for old, new in zip(seq[:-1], seq[1:]):
        a.switch(old, new)
        b.switch(old, new)
        ga, gb = a.rows(0), b.rows(0)
        assert (ga == gb).all()
        rep, _ = check_step(prev, gb, A, B, old, new)
        assert rep["fail"] == 0
        prev = gb
    a.close()
    b.close()


@pytest.mark.parametrize("variant", [2, 1])
def test_item_pool_against_the_static_split(variant):
    """With each XCD on its own eighth of the items (the resident-A kernel always; the streaming kernel, variant 1, where
    the host chooses that order or LSW_OPT_XCD_REMAP = 2 forces it) the kernel deals the last sixteenth of every XCD's items through an atomic pool counter
    (LSW_OPT_XCD_POOL, on by default) when a launch has enough items; 256-column items and a 64-workgroup grid make a
    42-million-weight stack qualify.  Every item must be taken exactly once (a second application of an in-place update
    would show), launch after launch (the kernel resets its own counters): same bits as the static split, and the
    oracle's bar."""
    E, r, grid = 4, 8, 64
    dims = [(2048, 2048), (4096, 1024), (1000, 2048), (3000, 512), (520, 2056), (1536, 1024),
            (4096, 2048), (130, 1032), (777, 1024), (2048, 2048), (8192, 1024), (2560, 2048)]
    rng = np.random.default_rng(9090)
    host = [I.host_linear(rng, o, n, E, r, 0.02, 1 / 16, 0.01) for o, n in dims]
    shapes = [(p // 3, p % 3, o, n) for p, (o, n) in enumerate(dims)]
    a = DeviceStack.from_host(host, shapes, E, r, kernel=L.KERNEL_MFMA)
    b = DeviceStack.from_host(host, shapes, E, r, kernel=L.KERNEL_MFMA)
    for ds in (a, b):
        L.lsw_set_option(ds.ctx, L.LSW_OPT_GRID, grid)
        L.lsw_set_option(ds.ctx, L.LSW_OPT_TILE_COLS, 256)
        if variant == 1:
            L.lsw_set_option(ds.ctx, L.LSW_OPT_RESIDENT_Q, 0)
            L.lsw_set_option(ds.ctx, L.LSW_OPT_XCD_REMAP, 2)
    L.lsw_set_option(b.ctx, L.LSW_OPT_XCD_POOL, 0)
    none = (np.zeros(0, np.int32), np.zeros(0, np.float32))
    seq = [none, (np.array([1, 2], np.int32), np.array([0.7, 0.3], np.float32)),
           (np.array([2, 0], np.int32), np.array([0.45, 0.55], np.float32)),
           (np.array([3, 1], np.int32), np.array([0.5, 0.5], np.float32)), none]
    prev = [a.rows(p) for p in range(len(dims))]

    def both(old, new, layers, expect_pool=True):
        a.switch(old, new, layers=layers)
        b.switch(old, new, layers=layers)
        assert L.lsw_query(a.ctx, L.LSW_Q_LAST_VARIANT) == variant and L.lsw_query(b.ctx, L.LSW_Q_LAST_VARIANT) == variant
        n_items = L.lsw_query(a.ctx, L.LSW_Q_LAST_ITEMS)
        per = -(-n_items // 8)
        if expect_pool:
            assert per // 16 > 0 and n_items - 7 * per - per // 16 >= 2 * (grid // 8), "this launch would not use the pool"
        for p, (layer, _, _, _) in enumerate(shapes):
            ga, gb = a.rows(p), b.rows(p)
            assert (ga == gb).all(), (layers, p)
            if layers is None or layer in layers:
                rep, _ = check_step(prev[p], ga, host[p][1], host[p][2], old, new)
                assert rep["fail"] == 0, (layers, p)
            else:
                assert (ga == prev[p]).all()
            prev[p] = ga

    both(seq[0], seq[1], None)
    both(seq[1], seq[2], None)
    both(seq[2], seq[3], [0, 2])          # subset launches (fewer items, other pool size) between full ones
    both(seq[2], seq[3], [1, 3])
    both(seq[3], seq[4], None)

    # the pool counters are reset by the kernel itself, so recorded launches replay correctly: merge and unmerge of one
    # set, each recorded once, replayed in turn, against the same switches launched eagerly with the static split
    graphs = []
    for old, new in ((seq[0], seq[1]), (seq[1], seq[0])):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            a.switch(old, new)                # recorded, not run
        graphs.append((g, old, new))
    for _ in range(2):
        for g, old, new in graphs:
            g.replay()
            b.switch(old, new)
            torch.cuda.synchronize()
            for p in range(len(dims)):
                assert (a.rows(p) == b.rows(p)).all(), p
    a.close()
    b.close()


@pytest.mark.parametrize("resident", [1, 0])
@pytest.mark.parametrize("group", [1, 3, 4])
def test_panel_groups_change_the_item_order_and_nothing_else(resident, group):
    """LSW_OPT_PANEL_GROUP takes the column panels of a wide matrix in groups (all row blocks of one group before the
    next); the launch must still touch every tile exactly once: same bits as the rows-outermost order, and the oracle's bar."""
    E, r = 4, 8
    dims = [(260, 4104), (520, 2056), (130, 256), (300, 1288)]          # 17, 9, 1 and 6 panels of 256 columns
    rng = np.random.default_rng(515 + group)
    host = [I.host_linear(rng, o, n, E, r, 0.02, 1 / 16, 0.01) for o, n in dims]
    shapes = [(0, p, o, n) for p, (o, n) in enumerate(dims)]
    a = DeviceStack.from_host(host, shapes, E, r, kernel=L.KERNEL_MFMA)
    b = DeviceStack.from_host(host, shapes, E, r, kernel=L.KERNEL_MFMA)
    for ds in (a, b):
        L.lsw_set_option(ds.ctx, L.LSW_OPT_TILE_COLS, 256)
        L.lsw_set_option(ds.ctx, L.LSW_OPT_RESIDENT_Q, resident)
        L.lsw_set_option(ds.ctx, L.LSW_OPT_XCD_REMAP, 2)
    L.lsw_set_option(a.ctx, L.LSW_OPT_PANEL_GROUP, group)
    L.lsw_set_option(b.ctx, L.LSW_OPT_PANEL_GROUP, 0)
    none = (np.zeros(0, np.int32), np.zeros(0, np.float32))
    seq = [none, (np.array([1, 2], np.int32), np.array([0.7, 0.3], np.float32)),
           (np.array([2, 0], np.int32), np.array([0.45, 0.55], np.float32)), none]
    prev = [a.rows(p) for p in range(len(dims))]
    for old, new in zip(seq[:-1], seq[1:]):
        a.switch(old, new)
        b.switch(old, new)
        for p in range(len(dims)):
            ga, gb = a.rows(p), b.rows(p)
            assert (ga == gb).all(), p
            rep, _ = check_step(prev[p], ga, host[p][1], host[p][2], old, new)
            assert rep["fail"] == 0, p
            prev[p] = ga
    a.close()
    b.close()


@pytest.mark.parametrize("kernel", KERNELS)
def test_stack_with_layer_subsets_guard_bands_and_state(kernel):
    wl = I.Workload("mini", 3, 64, 136, 32, 6, 8, 2, 4, 0.02, 1 / 8, 0.01, 4242)
    shapes = wl.linear_shapes()
    host = I.host_stack(wl)
    # every W sits inside a larger buffer with sentinel bands before and after it
    GUARD = 256
    dev, bufs = [], []
    for (W, A, B), (_, _, o, n) in zip(host, shapes):
        buf = torch.full((GUARD + o * n + GUARD,), -7.0, dtype=torch.bfloat16, device="cuda")
        view = buf[GUARD:GUARD + o * n].view(o, n)
        view.copy_(bits_to_device(W))
        bufs.append(buf)
        dev.append((view, torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()))
    ds = DeviceStack(dev, shapes, wl.experts, wl.rank, kernel=kernel)
    assert L.lsw_query(ds.ctx, L.LSW_Q_N_LINEARS) == 21 and L.lsw_query(ds.ctx, L.LSW_Q_N_LAYERS) == 3
    none = (np.zeros(0, np.int32), np.zeros(0, np.float32))
    a = (np.array([1, 4], np.int32), np.array([0.7, 0.3], np.float32))
    b = (np.array([4, 2], np.int32), np.array([0.55, 0.45], np.float32))
    prev = [ds.rows(p) for p in range(len(shapes))]

    def run(old, new, layers):
        ds.switch(old, new, layers=layers)
        for p, (layer, _, _, _) in enumerate(shapes):
            got = ds.rows(p)
            if layers is None or layer in layers:
                rep, _ = check_step(prev[p], got, host[p][1], host[p][2], old, new)
                assert rep["fail"] == 0, (p, layers)
                assert (got != prev[p]).mean() > 0.3
            else:
                assert (got == prev[p]).all(), f"linear {p} of an unselected layer changed"
            prev[p] = got

    run(none, a, None)
    run(a, b, [1])                       # only layer 1 moves to b (expert 4 is in both sets: 3 terms)
    assert L.lsw_get_state(ds.ctx, 1)[0].tolist() == [4, 2]
    assert L.lsw_get_state(ds.ctx, 0)[0].tolist() == [1, 4]
    run(a, b, [2, 0])                    # the other two follow
    run(b, none, None)
    for buf in bufs:
        assert (buf[:GUARD] == -7.0).all() and (buf[-GUARD:] == -7.0).all(), "guard band overwritten"

    # strict state: a wrong `old` is refused and nothing changes
    L.lsw_set_option(ds.ctx, L.LSW_OPT_STRICT_STATE, 1)
    with pytest.raises(L.LswError) as e:
        ds.switch(a, b)
    assert e.value.status == L.LSW_ERR_STATE
    for p in range(len(shapes)):
        assert (ds.rows(p) == prev[p]).all()
    ds.switch(none, a)                   # the true state (nothing merged) is accepted
    with pytest.raises(L.LswError) as e:
        ds.switch(none, a, layers=[7])
    assert e.value.status == L.LSW_ERR_ARG
    ds.close()


@pytest.mark.parametrize("kernel", KERNELS)
def test_invariants_on_device(kernel):
    rng = np.random.default_rng(9)
    W, A, B = I.host_linear(rng, 96, 520, 8, 8, 0.02, 1 / 16, 0.01)
    ds = DeviceStack.from_host([(W, A, B)], [(0, 0, 96, 520)], 8, 8, kernel=kernel)
    none = (np.zeros(0, np.int32), np.zeros(0, np.float32))
    s = (np.array([3, 5], np.int32), np.array([0.6, 0.4], np.float32))
    # k_old = k_new = 0: nothing is launched, W untouched
    ds.switch(none, none)
    assert L.lsw_query(ds.ctx, L.LSW_Q_LAST_KERNEL) == 0 and (ds.rows(0) == W).all()
    ds.switch(none, s)
    W1 = ds.rows(0)
    assert (W1 == O.switch_step(W, A, B, [], [], s[0], s[1])).mean() > 0.999
    # switching to the same set (any order): identical pairs cancel, no launch, bit-identical
    ds.switch(s, (s[0][::-1].copy(), s[1][::-1].copy()))
    assert L.lsw_query(ds.ctx, L.LSW_Q_LAST_KERNEL) == 0 and (ds.rows(0) == W1).all()
    # gates one fp32 ulp apart do not cancel: a launch happens and the 1-ulp rule holds
    s2 = (s[0], np.nextafter(s[1], np.float32(1.0)).astype(np.float32))
    ds.switch(s, s2)
    assert L.lsw_query(ds.ctx, L.LSW_Q_LAST_KERNEL) == kernel
    rep, _ = check_step(W1, ds.rows(0), A, B, s, s2)
    assert rep["fail"] == 0
    # merge then unmerge: the GPU agrees with the oracle on which elements return exactly
    W2p = ds.rows(0)
    ds.switch(s2, none)
    rep, want = check_step(W2p, ds.rows(0), A, B, s2, none)
    assert rep["fail"] == 0
    # bad arguments leave W untouched
    before = ds.rows(0)
    for old, new in [((np.array([1, 1], np.int32), np.array([.5, .5], np.float32)), none),
                     (none, (np.array([8], np.int32), np.array([1.0], np.float32))),
                     (none, (np.array([1], np.int32), np.array([np.nan], np.float32)))]:
        with pytest.raises(L.LswError) as e:
            ds.switch(old, new)
        assert e.value.status == L.LSW_ERR_ARG
    assert (ds.rows(0) == before).all()
    ds.close()


def test_merged_gemv_against_oracle():
    rng = np.random.default_rng(10)
    for out, inn in [(37, 264), (256, 4096), (100, 11008), (16, 8)]:
        W, A, B = I.host_linear(rng, out, inn, 2, 8, 0.02, 1 / 16, 0.01)
        ds = DeviceStack.from_host([(W, A, B)], [(0, 0, out, inn)], 2, 8)
        ds.switch((np.zeros(0, np.int32), np.zeros(0, np.float32)), (np.array([1], np.int32), np.array([1.0], np.float32)))
        x = I.f32_to_bf16_bits(rng.normal(0, 1, inn).astype(np.float32))
        xd = bits_to_device(x)
        y = torch.empty(out, dtype=torch.float32, device="cuda")
        L.lsw_merged_gemv(ds.ctx, 0, xd.data_ptr(), y.data_ptr(), torch.cuda.current_stream().cuda_stream)
        Wm = ds.rows(0)
        want = O.gemv(Wm, x)
        absum = np.abs(O.bf16_bits_to_f64(Wm)) @ np.abs(O.bf16_bits_to_f64(x))
        err = np.abs(y.cpu().numpy().astype(np.float64) - want)
        assert (err <= 1e-5 * absum + 1e-30).all(), (out, inn, float((err / absum).max()))
        ds.close()


def test_merged_decode_after_many_switches_stays_within_the_predicted_drift():
    """Eq. 2 == Eq. 3 after T free-running switches: decode through the merged weights against W0 x + sum_c g_c B_c (A_c x)
    in fp64 from the BASE weights.  They differ by the rounding drift of the merged weights alone: per weight a random
    walk of about 0.29 * sqrt(T) ulp, so |err_i| is about 0.29 * sqrt(T) * 2^-8 * sqrt(sum_j W_ij^2 x_j^2); gated at 6x."""
    wl = I.Workload("mini", 1, 256, 520, 64, 8, 8, 2, 24, 0.02, 1 / 16, 0.01, 4246)
    host = I.host_stack(wl)
    ds = DeviceStack.from_host(host, wl.linear_shapes(), wl.experts, wl.rank)
    routes = _route_stream(wl, wl.steps)
    old = (np.zeros(0, np.int32), np.zeros(0, np.float32))
    for new in routes:
        ds.switch(old, new)
        old = new
    rng = np.random.default_rng(12)
    worst = 0.0
    for p, (W0, A, B) in enumerate(host):
        out, inn = W0.shape
        x = I.f32_to_bf16_bits(rng.normal(0, 1, inn).astype(np.float32))
        y = torch.empty(out, dtype=torch.float32, device="cuda")
        L.lsw_merged_gemv(ds.ctx, p, bits_to_device(x).data_ptr(), y.data_ptr(), torch.cuda.current_stream().cuda_stream)
        xv, w0 = O.bf16_bits_to_f64(x), O.bf16_bits_to_f64(W0)
        want = w0 @ xv + O.gated_lowrank_sum(A, B, old[0], old[1]) @ xv
        wm = O.bf16_bits_to_f64(ds.rows(p))
        predicted = 0.29 * np.sqrt(wl.steps) * 2.0 ** -8 * np.sqrt((wm ** 2) @ (xv ** 2))
        err = np.abs(y.cpu().numpy().astype(np.float64) - want)
        assert (err <= 6 * predicted + 1e-5 * (np.abs(wm) @ np.abs(xv))).all(), (p, float((err / predicted).max()))
        worst = max(worst, float(np.median(err / predicted)))
        assert np.median(err / predicted) > 0.2, "the drift should be visible: it is what lsw_rebase removes"
    print(f"\n[merged decode after {wl.steps} switches] median error / predicted drift up to {worst:.2f}")
    ds.close()


def test_merged_gemv_all_linears_in_one_launch():
    """Every linear of a small ragged stack decoded by ONE launch; each output row against the fp64 oracle."""
    rng = np.random.default_rng(11)
    dims = [(37, 264), (5, 8), (130, 1032), (64, 4096), (3, 11008), (258, 520)]
    host = [I.host_linear(rng, o, n, 2, 8, 0.02, 1 / 16, 0.01) for o, n in dims]
    shapes = [(p // 3, p % 3, o, n) for p, (o, n) in enumerate(dims)]
    ds = DeviceStack.from_host(host, shapes, 2, 8)
    ds.switch((np.zeros(0, np.int32), np.zeros(0, np.float32)), (np.array([0], np.int32), np.array([1.0], np.float32)))
    assert L.lsw_query(ds.ctx, L.LSW_Q_GEMV_X_ELEMS) == sum(n for _, n in dims)
    assert L.lsw_query(ds.ctx, L.LSW_Q_GEMV_Y_ELEMS) == sum(o for o, _ in dims)
    xs = [I.f32_to_bf16_bits(rng.normal(0, 1, n).astype(np.float32)) for _, n in dims]
    xd = bits_to_device(np.concatenate(xs))
    guard = 16
    y = torch.full((sum(o for o, _ in dims) + guard,), 7.5, dtype=torch.float32, device="cuda")
    for grid in (0, 8, 64):
        L.lsw_set_option(ds.ctx, L.LSW_OPT_GEMV_GRID, grid)
        y.fill_(7.5)
        L.lsw_merged_gemv_all(ds.ctx, xd.data_ptr(), y.data_ptr(), torch.cuda.current_stream().cuda_stream)
        got = y.cpu().numpy().astype(np.float64)
        assert (got[-guard:] == 7.5).all()
        at = 0
        for p, (o, n) in enumerate(dims):
            Wm = ds.rows(p)
            want = O.gemv(Wm, xs[p])
            absum = np.abs(O.bf16_bits_to_f64(Wm)) @ np.abs(O.bf16_bits_to_f64(xs[p]))
            err = np.abs(got[at:at + o] - want)
            assert (err <= 1e-5 * absum + 1e-30).all(), (grid, p, o, n, float((err / absum).max()))
            at += o
    ds.close()


def test_matrix_loop_probe_reports_a_plausible_rate():
    ns = L.lsw_probe_matrix_loop(50, 2, 2, False)
    ns0 = L.lsw_probe_matrix_loop(50, 2, 0, True)
    # 192 matrix-pipe cycles per group: 80 ns at the 2.4 GHz peak clock; anything far outside is a broken probe
    assert 60.0 < ns0 < 400.0 and 60.0 < ns < 400.0 and ns0 <= ns * 1.1, (ns0, ns)
    for bad in ((0, 1, 0), (10, 0, 0), (10, 1, 3)):
        with pytest.raises(L.LswError):
            L.lsw_probe_matrix_loop(bad[0], bad[1], bad[2], False)


def test_probe_inplace_leaves_weights_unchanged():
    wl = I.Workload("mini", 2, 64, 136, 32, 4, 8, 2, 4, 0.02, 1 / 8, 0.01, 515)
    host = I.host_stack(wl)
    ds = DeviceStack.from_host(host, wl.linear_shapes(), wl.experts, wl.rank)
    for wpc in (1, 4, 0):          # 0 = the switch kernel's own launch with the work taken out
        L.lsw_probe_inplace(ds.ctx, wpc, torch.cuda.current_stream().cuda_stream)
    for p_, (W, _, _) in enumerate(host):
        got = ds.rows(p_)
        neg_zero = W == 0x8000
        assert (got[~neg_zero] == W[~neg_zero]).all()
        assert (got[neg_zero] == 0).all()
    for bad in (-1, 17):
        with pytest.raises(L.LswError):
            L.lsw_probe_inplace(ds.ctx, bad)
    ds.close()
