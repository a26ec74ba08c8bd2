"""GPU parity at full workload shapes, in the launch configuration bench.py times.

The 7B-shaped stack (32 layers x 7 linears, 6.48e9 weights) is switched 64 times; on steps
1, 2, 3, 32 and 64 sampled rows of EVERY linear are compared, teacher-forced, with the oracle
(elements are independent, so sampling rows is sound), and two whole linears are compared in
full at step 1.  The 13B-, 70B- and rank-64 stacks run the same way at their full size for a few steps
(fewer sampled rows), and on a reduced layer count for more steps."""
import os

import numpy as np
import pytest
import torch

from oracle import lsw_oracle as O
from paper_2405_17741_amd import binding as L
from paper_2405_17741_amd import inputs as I
from tests.gpu_harness import DeviceStack, check_step, gate_quality, merge_reports

pytestmark = pytest.mark.gpu
NONE = (np.zeros(0, np.int32), np.zeros(0, np.float32))


def _run_sampled(wl, check_steps, full_linears=(), n_random_rows=61, kernel=L.KERNEL_AUTO, factor_dtype=torch.float32,
                 device_routed=False, ld_of=None):
    """factor_dtype bf16: the factors are stored as bf16 (the oracle gets exactly those values).  device_routed: every
    token's (ids, gates) comes from lsw_route_dev and stays on the device, the switch is lsw_switch_dev (term list built
    on the device, launches sized for k_old + k_new terms); ids must equal the oracle router's, the gates it produced are
    what the oracle's switch is given."""
    shapes = wl.linear_shapes()
    stack = I.device_stack(wl, factor_dtype=factor_dtype, ld_of=ld_of)      # ld_of: weights stored at a leading dimension > in
    ds = DeviceStack(stack, shapes, wl.experts, wl.rank, kernel=kernel)
    rng = np.random.default_rng(wl.seed + 1)
    rows = [I.sample_rows(rng, o, n_random_rows) for _, _, o, _ in shapes]
    A_host = [A.float().cpu().numpy() for _, A, _ in stack]
    B_rows = [B.index_select(1, torch.as_tensor(r, device=B.device)).float().cpu().numpy() for (_, _, B), r in zip(stack, rows)]
    logits = I.router_logits(wl)
    routes = [O.route(l, wl.top_k) for l in logits]
    stream = torch.cuda.current_stream().cuda_stream
    if device_routed:
        logits_d = torch.from_numpy(logits.copy()).cuda()
        bufs = [(torch.zeros(wl.top_k, dtype=torch.int32, device="cuda"), torch.zeros(wl.top_k, dtype=torch.float32, device="cuda"))
                for _ in range(2)]
    old = NONE
    reports, kernels = [], set()
    for t, new in enumerate(routes, start=1):
        checked = t in check_steps
        if checked:
            before = [ds.rows(p, rows[p]) for p in range(len(shapes))]
            full_before = {p: ds.rows(p) for p in full_linears} if t == 1 else {}
        if device_routed:
            (oi, og), (ni, ng) = bufs[t % 2], bufs[(t + 1) % 2]
            L.lsw_route_dev(ds.ctx, logits_d[t - 1].data_ptr(), wl.top_k, ni.data_ptr(), ng.data_ptr(), stream)
            L.lsw_switch_dev(ds.ctx, oi.data_ptr(), og.data_ptr(), 0 if t == 1 else wl.top_k, ni.data_ptr(), ng.data_ptr(), wl.top_k,
                             stream=stream)
            assert ni.cpu().numpy().tolist() == new[0].tolist(), t           # the selection: bit-exact
            new = (new[0], ng.cpu().numpy().copy())                          # the device router's own gates
        else:
            ds.switch(old, new)
        kernels.add(L.lsw_query(ds.ctx, L.LSW_Q_LAST_KERNEL))
        if checked:
            step_reports = []
            for p in range(len(shapes)):
                got = ds.rows(p, rows[p])
                # B_rows already holds only the sampled rows, so the oracle sees a [len(rows), in] problem
                rep, _ = check_step(before[p], got, A_host[p], B_rows[p], old, new)
                assert rep["fail"] == 0, (wl.name, t, p, {k: v for k, v in rep.items() if k != "fail_mask"})
                step_reports.append(rep)
            for p, wb in full_before.items():
                Bf = stack[p][2].cpu().numpy()
                rep, _ = check_step(wb, ds.rows(p), A_host[p], Bf, old, new)
                assert rep["fail"] == 0, (wl.name, "full", p)
                step_reports.append(rep)
            tot = merge_reports(step_reports)
            print(f"[{wl.name} step {t}] n={tot['n']} exact={tot['exact_frac']:.6f} "
                  f"clause2={tot['needed_clause2']} maxdist={tot['max_dist']} kernels={sorted(kernels)}", flush=True)
            gate_quality(tot, f"{wl.name} step {t}", rank=wl.rank)
            reports.append(tot)
        old = new
    if device_routed:
        assert L.lsw_dev_status(ds.ctx) == 0
    torch.cuda.synchronize()
    for (W, _, _), (_, _, _, n_cols) in zip(stack, shapes):          # padding columns (if any) still hold their guard value
        if W._base is not None and W._base.shape[1] > n_cols:
            assert bool((W._base[:, n_cols:] == I.PAD_GUARD).all()), "padding columns were written"
    ds.close()
    return reports, kernels


def test_7b_full_size_sampled_rows_every_linear():
    wl = I.WORKLOADS["7b"]
    rng = np.random.default_rng(7)
    full = (int(rng.integers(0, 32)) * 7 + 0, int(rng.integers(0, 32)) * 7 + 4)   # one 4096x4096, one 11008x4096
    reports, kernels = _run_sampled(wl, {1, 2, 3, 32, 64}, full_linears=full)
    assert kernels <= {L.KERNEL_MFMA}
    assert len(reports) == 5


def test_7b_full_size_factors_stored_as_bf16():
    """The launch configuration `bench.py --factor-dtype bf16` times: the streaming kernel, each XCD on its own eighth of the
    items, the tail of every eighth dealt through the pool."""
    wl = I.Workload(**{**I.WORKLOADS["7b"].__dict__, "steps": 8})
    reports, kernels = _run_sampled(wl, {1, 2, 8}, n_random_rows=13, factor_dtype=torch.bfloat16)
    assert kernels == {L.KERNEL_MFMA}
    assert len(reports) == 3


def test_7b_full_size_at_a_fast_row_pitch():
    """The launch configuration of bench.py's 7b_pitch_padded entry: every weight whose rows are not 4, 8, 16 or 32 KB apart
    (the 32 `down` matrices, 11008 columns) stored at the next such leading dimension; sampled rows of every linear against
    the oracle, and every padding column untouched at the end."""
    wl = I.Workload(**{**I.WORKLOADS["7b"].__dict__, "steps": 8})
    pitch = lambda n: next(p for p in (2048, 4096, 8192, 16384) if p >= n) if n <= 16384 else n
    reports, kernels = _run_sampled(wl, {1, 2, 3, 8}, n_random_rows=13, ld_of=pitch)
    assert kernels == {L.KERNEL_MFMA}
    assert len(reports) == 4


def test_7b_full_size_device_routed_token_steps():
    """lsw_route_dev + lsw_switch_dev over the whole stack: the kernels are sized for four terms and read a list of three
    or four from device memory."""
    wl = I.Workload(**{**I.WORKLOADS["7b"].__dict__, "steps": 8})
    reports, kernels = _run_sampled(wl, {1, 2, 3, 8}, n_random_rows=13, device_routed=True)
    assert kernels == {L.KERNEL_MFMA}
    assert len(reports) == 4


def _twin_stacks_stay_identical(wl, options_b, steps):
    """Two copies of a stack, the second with other launch options (item order, pool, kernel choice): the orders differ,
    the arithmetic per element does not, so after every switch EVERY weight must hold the same bits.  A skipped item or
    one applied twice anywhere in the launch shows."""
    shapes = wl.linear_shapes()
    a = DeviceStack(I.device_stack(wl), shapes, wl.experts, wl.rank)
    b = DeviceStack(I.device_stack(wl), shapes, wl.experts, wl.rank)
    for opt, value in options_b:
        L.lsw_set_option(b.ctx, opt, value)
    routes = [O.route(l, wl.top_k) for l in I.router_logits(wl, steps)]
    old = NONE
    variants = set()
    for t, new in enumerate(routes, start=1):
        a.switch(old, new)
        b.switch(old, new)
        variants.add((L.lsw_query(a.ctx, L.LSW_Q_LAST_VARIANT), L.lsw_query(b.ctx, L.LSW_Q_LAST_VARIANT)))
        for p in range(len(shapes)):
            assert torch.equal(a.stack[p][0].view(torch.int16), b.stack[p][0].view(torch.int16)), (wl.name, t, p)
        old = new
    a.close()
    b.close()
    return variants


def test_7b_full_size_pool_and_kernel_choice_leave_the_same_bits_for_64_switches():
    """The headline launch (A resident in LDS, per-XCD order, item pool) against the streaming kernel in the round-wise
    order on a second copy of the whole stack: all 6.5e9 weights compared after each of 64 switches."""
    wl = I.WORKLOADS["7b"]
    variants = _twin_stacks_stay_identical(wl, [(L.LSW_OPT_RESIDENT_Q, 0), (L.LSW_OPT_XCD_REMAP, 1)], wl.steps)
    assert variants == {(2, 1)}


def test_70b_shape_forty_layers_item_order_leaves_the_same_bits():
    """Half the 70B-shaped stack twice (2 x 68 GB): per-XCD order with the pool and panel groups against the round-wise
    order with rows outermost."""
    free, _ = torch.cuda.mem_get_info()
    if free < 170e9:
        pytest.skip("needs 170 GB of free device memory")
    wl = I.scaled(I.WORKLOADS["70b"], 40)
    variants = _twin_stacks_stay_identical(wl, [(L.LSW_OPT_XCD_REMAP, 1), (L.LSW_OPT_PANEL_GROUP, 0), (L.LSW_OPT_RESIDENT_Q, 0)], 5)
    assert {v[1] for v in variants} == {1}


def test_13b_shape_with_forced_reuse_two_layers():
    wl = I.scaled(I.WORKLOADS["13b"], 2)
    reports, kernels = _run_sampled(wl, {1, 2, 3, 17, 33, 64}, n_random_rows=29)
    assert L.KERNEL_MFMA in kernels
    # the stream really reuses experts: some steps have 3 terms (one id in both sets)
    routes = [O.route(l, 2)[0].tolist() for l in I.router_logits(wl)]
    reuse = sum(len(set(a) & set(b)) > 0 for a, b in zip(routes[:-1], routes[1:]))
    assert 20 <= reuse <= 50


def test_70b_shape_one_layer():
    wl = I.scaled(I.WORKLOADS["70b"], 1)
    wl = I.Workload(**{**wl.__dict__, "steps": 4})
    reports, kernels = _run_sampled(wl, {1, 2, 4}, n_random_rows=13)
    assert kernels == {L.KERNEL_MFMA}


def test_7b_rank64_one_layer():
    wl = I.scaled(I.WORKLOADS["7b_r64"], 1)
    wl = I.Workload(**{**wl.__dict__, "steps": 3})
    reports, kernels = _run_sampled(wl, {1, 2, 3}, n_random_rows=13)
    assert kernels == {L.KERNEL_MFMA}          # fused ranks 64..256: the chunked matrix-core kernel


def test_13b_full_size_sampled_rows_every_linear():
    """All 40 layers of the 13B-shaped stack (12.7e9 weights, every row pitch off the fast ones, forced expert reuse)."""
    wl = I.Workload(**{**I.WORKLOADS["13b"].__dict__, "steps": 6})
    reports, kernels = _run_sampled(wl, {1, 2, 6}, n_random_rows=13)
    assert kernels == {L.KERNEL_MFMA}
    assert len(reports) == 3


def test_13b_full_size_at_a_fast_row_pitch():
    """bench.py's 13b_pitch_padded entry: all 40 layers with every weight at a leading dimension of 8192 or 16384 elements (38 GB
    allocated for 25 GB of weights); sampled rows against the oracle, every padding column untouched."""
    wl = I.Workload(**{**I.WORKLOADS["13b"].__dict__, "steps": 3})
    pitch = lambda n: next(p for p in (2048, 4096, 8192, 16384) if p >= n) if n <= 16384 else n
    reports, kernels = _run_sampled(wl, {1, 2, 3}, n_random_rows=13, ld_of=pitch)
    assert kernels == {L.KERNEL_MFMA}
    assert len(reports) == 3


def test_7b_rank64_full_size_sampled_rows_every_linear():
    """All 32 layers with rank-64 experts: the chunked matrix-core kernel over the whole stack."""
    wl = I.Workload(**{**I.WORKLOADS["7b_r64"].__dict__, "steps": 3})
    reports, kernels = _run_sampled(wl, {1, 2, 3}, n_random_rows=13)
    assert kernels == {L.KERNEL_MFMA}
    assert len(reports) == 3


def test_70b_full_size_sampled_rows_every_linear():
    """All 80 layers of the 70B-shaped stack: 68.5e9 weights (137 GB) in one launch, element offsets far beyond 32 bits
    across the stack, 4.2 million work items."""
    free, _ = torch.cuda.mem_get_info()
    if free < 160e9:
        pytest.skip("needs 160 GB of free device memory")
    wl = I.Workload(**{**I.WORKLOADS["70b"].__dict__, "steps": 2})
    reports, kernels = _run_sampled(wl, {1, 2}, n_random_rows=5)
    assert kernels == {L.KERNEL_MFMA}
    assert len(reports) == 2
