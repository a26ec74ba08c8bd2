"""Weights stored at a leading dimension larger than their row length (lsw_linear::ld): every kernel family must give
the bits it gives on the dense matrix, meet the bar against the oracle, and never touch the padding columns."""
import numpy as np
import pytest
import torch

from oracle import lsw_oracle as O
from paper_2405_17741_amd import binding as L
from paper_2405_17741_amd import inputs as I
from tests.gpu_harness import DeviceStack, bits_to_device, check_step, device_to_bits

pytestmark = pytest.mark.gpu
NONE = (np.zeros(0, np.int32), np.zeros(0, np.float32))
GUARD = 0xC0F0          # bf16 -7.5: what the padding holds


def _padded(W_bits, ld):
    out, inn = W_bits.shape
    full = np.full((out, ld), GUARD, np.uint16)
    full[:, :inn] = W_bits
    dev = bits_to_device(full)
    return dev, dev[:, :inn]


CASES = [
    # out, in, ld, E, r, kernel option, resident-A option, terms
    (100, 264, 272, 5, 8, L.KERNEL_VALU, 1, 3),
    (130, 1000, 2048, 6, 8, L.KERNEL_MFMA, 1, 4),        # A resident in LDS; rows 4 KB apart
    (130, 1000, 1008, 6, 8, L.KERNEL_MFMA, 0, 4),        # A streamed per step
    (260, 4104, 4360, 4, 16, L.KERNEL_MFMA, 1, 4),       # fused rank 64, several items per row block, ragged last item
    (129, 520, 776, 4, 32, L.KERNEL_MFMA, 1, 4),         # fused rank 128: the chunked kernel
    (37, 8, 16, 5, 8, L.KERNEL_MFMA, 1, 2),
    (65, 136, 144, 3, 4, L.KERNEL_VALU, 1, 2),
]


@pytest.mark.parametrize("case", CASES)
def test_switch_on_a_padded_weight_equals_the_dense_one(case):
    out, inn, ld, E, r, kernel, resident, n_terms = case
    rng = np.random.default_rng(out * 31 + inn + ld)
    W, A, B = I.host_linear(rng, out, inn, E, r, 0.02, 1 / 16, 0.01)
    Ad, Bd = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    full, view = _padded(W, ld)
    dense = DeviceStack.from_host([(W, A, B)], [(0, 0, out, inn)], E, r, kernel=kernel)
    padded = DeviceStack([(view, Ad, Bd)], [(0, 0, out, inn)], E, r, kernel=kernel)
    for ds in (dense, padded):
        L.lsw_set_option(ds.ctx, L.LSW_OPT_RESIDENT_Q, resident)
    k = n_terms // 2
    sets = [(rng.choice(E, k, replace=False).astype(np.int32), rng.random(k).astype(np.float32)) for _ in range(3)]
    seq = [NONE] + sets + [NONE]
    prev = W
    for old, new in zip(seq[:-1], seq[1:]):
        dense.switch(old, new)
        padded.switch(old, new)
        assert L.lsw_query(dense.ctx, L.LSW_Q_LAST_VARIANT) == L.lsw_query(padded.ctx, L.LSW_Q_LAST_VARIANT)
        got = device_to_bits(full)
        assert (got[:, inn:] == GUARD).all(), "padding columns must never be written"
        assert (got[:, :inn] == dense.rows(0)).all(), "same arithmetic as on the dense matrix"
        rep, _ = check_step(prev, got[:, :inn].copy(), A, B, old, new)
        assert rep["fail"] == 0
        prev = got[:, :inn].copy()
    dense.close()
    padded.close()


def test_decode_rebase_and_probe_on_padded_weights():
    E, r = 4, 8
    shapes = [(0, 0, 200, 520), (0, 1, 64, 1032), (1, 0, 33, 264)]
    lds = [1024, 1040, 272]
    rng = np.random.default_rng(99)
    host = [I.host_linear(rng, o, n, E, r, 0.02, 1 / 16, 0.01) for _, _, o, n in shapes]
    bufs = [_padded(W, ld) for (W, _, _), ld in zip(host, lds)]
    bases = [_padded(W, ld) for (W, _, _), ld in zip(host, lds)]
    stack = [(view, torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()) for (_, view), (_, A, B) in zip(bufs, host)]
    ds = DeviceStack(stack, shapes, E, r)
    stream = torch.cuda.current_stream().cuda_stream
    a = (np.array([2, 0], np.int32), np.array([0.625, 0.375], np.float32))
    ds.switch(NONE, a)
    # merged decode through the padded weights, one linear and all at once
    xs = [I.f32_to_bf16_bits(rng.normal(0, 1, n).astype(np.float32)) for _, _, _, n in shapes]
    xd = bits_to_device(np.concatenate(xs))
    y_all = torch.zeros(sum(o for _, _, o, _ in shapes), dtype=torch.float32, device="cuda")
    L.lsw_merged_gemv_all(ds.ctx, xd.data_ptr(), y_all.data_ptr(), stream)
    at = 0
    for p, (_, _, o, n) in enumerate(shapes):
        Wm = device_to_bits(bufs[p][0])[:, :n].copy()
        want = O.gemv(Wm, xs[p])
        absum = np.abs(O.bf16_bits_to_f64(Wm)) @ np.abs(O.bf16_bits_to_f64(xs[p]))
        y1 = torch.zeros(o, dtype=torch.float32, device="cuda")
        L.lsw_merged_gemv(ds.ctx, p, bits_to_device(xs[p]).data_ptr(), y1.data_ptr(), stream)
        for got in (y_all[at:at + o].cpu().numpy().astype(np.float64), y1.cpu().numpy().astype(np.float64)):
            assert (np.abs(got - want) <= 1e-5 * absum + 1e-30).all(), p
        at += o
    # the probes rewrite every value as it is and leave the padding alone
    before = [device_to_bits(full) for full, _ in bufs]
    for wpc in (0, 2):
        L.lsw_probe_inplace(ds.ctx, wpc, stream)
    for (full, _), b in zip(bufs, before):
        assert (device_to_bits(full) == b).all()
    # re-base from padded base copies: with a set, and with none (the copy kernel)
    L.lsw_set_base(ds.ctx, [full.data_ptr() for full, _ in bases])
    b = (np.array([1, 3], np.int32), np.array([0.25, 0.75], np.float32))
    L.lsw_rebase(ds.ctx, b[0], b[1], stream=stream)
    for p, ((full, _), (W, A, B), (_, _, o, n)) in enumerate(zip(bufs, host, shapes)):
        got = device_to_bits(full)
        assert (got[:, n:] == GUARD).all()
        rep, _ = check_step(W, got[:, :n].copy(), A, B, NONE, b)
        assert rep["fail"] == 0, p
    L.lsw_rebase(ds.ctx, NONE[0], NONE[1], layers=[0], stream=stream)
    for p, ((full, _), (W, _, _), (layer, _, o, n)) in enumerate(zip(bufs, host, shapes)):
        got = device_to_bits(full)
        assert (got[:, n:] == GUARD).all()
        if layer == 0:
            assert (got[:, :n] == W).all(), "the base weights, bit for bit"
        else:
            assert (got[:, :n] != W).any()
    for full, _ in bases:
        assert (device_to_bits(full)[:, -1] == GUARD).all()
    ds.close()


def test_bad_leading_dimensions_are_refused():
    W = torch.zeros(64, 72, dtype=torch.bfloat16, device="cuda")
    A = torch.zeros(2, 8, 64, device="cuda")
    B = torch.zeros(2, 64, 8, device="cuda")
    for ld in (56, 68, 63):
        with pytest.raises(L.LswError) as e:
            L.lsw_create_adapters([(W.data_ptr(), A.data_ptr(), B.data_ptr(), 64, 64, 0, 0, ld)], 2, 8)
        assert e.value.status == L.LSW_ERR_SHAPE
    ctx = L.lsw_create_adapters([(W.data_ptr(), A.data_ptr(), B.data_ptr(), 64, 64, 0, 0, 72)], 2, 8)
    L.lsw_destroy(ctx)
