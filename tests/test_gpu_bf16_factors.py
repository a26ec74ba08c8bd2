"""GPU parity of the switch with the LoRA factors stored as bf16 (lsw_create_adapters_ex, LSW_FACTOR_BF16).

The update is defined on the stored values: the oracle gets the same bf16 values widened to fp32 and applies the
same formula in fp64, so the bar is the one of the fp32-factor tests (1 bf16 ulp, teacher-forced)."""
import numpy as np
import pytest
import torch

from oracle import lsw_oracle as O
from paper_2405_17741_amd import binding as L
from paper_2405_17741_amd import inputs as I
from tests.gpu_harness import bf16_factor_stack, DeviceStack, check_step, gate_quality, merge_reports

pytestmark = pytest.mark.gpu
NONE = (np.zeros(0, np.int32), np.zeros(0, np.float32))

SHAPES = [
    # out, in, E, r
    (37, 8, 5, 8), (100, 264, 5, 8), (64, 1048, 4, 16), (130, 520, 6, 24), (1, 16, 2, 8), (96, 256, 8, 32),
    # fused ranks above 64: the chunked kernel with 2, 3 and 4 chunks per step
    (150, 776, 5, 64), (129, 264, 4, 32), (33, 4360, 4, 48), (260, 520, 6, 40),
]


def _sequence(rng, E, r, steps=6):
    seq = [NONE]
    kmax = min(E, 2 if r > 16 else 3)
    for _ in range(steps):
        k = int(rng.integers(1, kmax + 1))
        ids = rng.choice(E, k, replace=False).astype(np.int32)
        g = rng.random(k).astype(np.float32)
        seq.append((ids, (g / g.sum()).astype(np.float32)))
    seq.append(NONE)
    return seq


@pytest.mark.parametrize("kernel", [L.KERNEL_VALU, L.KERNEL_MFMA, "mfma-two-pass"])
@pytest.mark.parametrize("shape", SHAPES)
def test_bf16_factors_ragged_shapes(shape, kernel):
    out, inn, E, r = shape
    two_pass = kernel == "mfma-two-pass"      # ranks that are multiples of 16 run one pass above 64 fused ranks by default
    if two_pass:
        if r < 32 or r % 16:
            pytest.skip("the one-pass mode does not apply to this rank")
        kernel = L.KERNEL_MFMA
    rng = np.random.default_rng(out * 977 + inn + r)
    host = bf16_factor_stack([I.host_linear(rng, out, inn, E, r, 0.02, 1 / 16, 0.01)])
    (W, A, B), = host
    ds = DeviceStack.from_host(host, [(0, 0, out, inn)], E, r, scale=0.5, bf16_factors=True)
    if two_pass:
        L.lsw_set_option(ds.ctx, L.LSW_OPT_ONE_PASS, 0)
    prev = ds.rows(0)
    reports, used = [], set()
    seq = _sequence(rng, E, r)
    for old, new in zip(seq[:-1], seq[1:]):
        n_terms = len(L.lsw_build_terms(old[0], old[1], new[0], new[1], E, 0.5)[0])
        fits = n_terms * (r // 8) <= 32
        L.lsw_set_option(ds.ctx, L.LSW_OPT_KERNEL, kernel if (kernel == L.KERNEL_VALU or fits) else L.KERNEL_VALU)
        ds.switch(old, new)
        used.add(L.lsw_query(ds.ctx, L.LSW_Q_LAST_KERNEL))
        got = ds.rows(0)
        rep, _ = check_step(prev, got, A, B, old, new, scale=0.5)
        assert rep["fail"] == 0, (old, new, {k: v for k, v in rep.items() if k != "fail_mask"})
        reports.append(rep)
        prev = got
    gate_quality(merge_reports(reports), f"bf16 factors ragged {shape} kernel={kernel}", exact_min=0.999, clause2_max=1.5e-4)
    if kernel == L.KERNEL_MFMA and r >= 32:
        assert L.KERNEL_MFMA in used
    ds.close()


def test_bf16_factors_equal_fp32_factors_holding_the_same_values():
    """The same values stored as fp32 and as bf16 define the same update: both contexts must pass the oracle check on
    the same W history, and the two results may differ only where the oracle's 1-ulp band allows."""
    wl = I.Workload("mini", 2, 64, 136, 32, 6, 8, 2, 4, 0.02, 1 / 8, 0.01, 777)
    shapes = wl.linear_shapes()
    host = bf16_factor_stack(I.host_stack(wl))
    a = DeviceStack.from_host(host, shapes, wl.experts, wl.rank, bf16_factors=True)
    b = DeviceStack.from_host(host, shapes, wl.experts, wl.rank)
    s1 = (np.array([1, 4], np.int32), np.array([0.7, 0.3], np.float32))
    s2 = (np.array([4, 2], np.int32), np.array([0.55, 0.45], np.float32))
    differ = total = 0
    for old, new in [(NONE, s1), (s1, s2), (s2, NONE)]:
        prev = [a.rows(p) for p in range(len(shapes))]
        for p in range(len(shapes)):       # keep both stacks on the same history
            b.stack[p][0].copy_(a.stack[p][0])
        a.switch(old, new)
        b.switch(old, new)
        for p in range(len(shapes)):
            ga, gb = a.rows(p), b.rows(p)
            for got in (ga, gb):
                rep, _ = check_step(prev[p], got, host[p][1], host[p][2], old, new)
                assert rep["fail"] == 0
            differ += int((ga != gb).sum())
            total += ga.size
    print(f"\n[bf16 vs fp32 storage of the same values] {differ} of {total} elements differ")
    assert differ <= 2e-4 * total
    a.close()
    b.close()


def test_bf16_factors_tiny_workload_every_step():
    wl = I.WORKLOADS["tiny"]
    host = bf16_factor_stack(I.host_stack(wl))
    (W0, A, B), = host
    ds = DeviceStack.from_host(host, wl.linear_shapes(), wl.experts, wl.rank, bf16_factors=True)
    routes = [O.route(l, wl.top_k) for l in I.router_logits(wl, wl.steps)]
    old, prev, reports = NONE, ds.rows(0), []
    for new in routes:
        ds.switch(old, new)
        got = ds.rows(0)
        rep, _ = check_step(prev, got, A, B, old, new)
        assert rep["fail"] == 0
        reports.append(rep)
        prev, old = got, new
    gate_quality(merge_reports(reports), "bf16 factors tiny", exact_min=0.999, clause2_max=1.5e-4)
    ds.close()


def test_create_ex_rejects_what_it_documents():
    W = torch.zeros(16, 16, dtype=torch.bfloat16, device="cuda")
    A = torch.zeros(2, 4, 16, dtype=torch.bfloat16, device="cuda")
    B = torch.zeros(2, 16, 4, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(L.LswError) as e:
        L.lsw_create_adapters([(W.data_ptr(), A.data_ptr(), B.data_ptr(), 16, 16, 0, 0)], 2, 4, 1.0, L.LSW_FACTOR_BF16)
    assert e.value.status == L.LSW_ERR_SHAPE
