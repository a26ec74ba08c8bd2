"""Device-resident routing: lsw_route_dev / lsw_switch_dev against the oracle and against the host-side path.

The token's (ids, gates) never visit the host on this path, so the tests check (1) the device router
against the oracle's router (ids bit for bit, gates to one fp32 ulp), (2) that a switch driven by device
lists leaves exactly the bits the host-driven switch leaves (same kernels, same coefficient arithmetic),
(3) the oracle, teacher-forced, on the device path, (4) what the device must refuse, and (5) a recorded
HIP graph of two token steps replayed with fresh logits against the same steps run eagerly."""
import numpy as np
import pytest
import torch

from oracle import lsw_oracle as O
from paper_2405_17741_amd import binding as L
from paper_2405_17741_amd import inputs as I
from tests.gpu_harness import DeviceStack, check_step

pytestmark = pytest.mark.gpu
NONE = (np.zeros(0, np.int32), np.zeros(0, np.float32))


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _dev_lists(ids, gates):
    return (torch.from_numpy(np.asarray(ids, np.int32)).cuda(), torch.from_numpy(np.asarray(gates, np.float32)).cuda())


def _f32_ulp_distance(a, b):
    ka = np.asarray(a, np.float32).view(np.int32).astype(np.int64)
    kb = np.asarray(b, np.float32).view(np.int32).astype(np.int64)
    return np.abs(ka - kb)


def _tiny_stack(kernel=L.KERNEL_AUTO):
    wl = I.WORKLOADS["tiny"]
    host = I.host_stack(wl)
    return wl, host, DeviceStack.from_host(host, wl.linear_shapes(), wl.experts, wl.rank, kernel=kernel)


def test_route_dev_matches_oracle_router():
    rng = np.random.default_rng(21)
    for E, k in [(8, 2), (8, 1), (16, 2), (16, 8), (100, 4), (3, 3), (4096, 8)]:
        W = torch.zeros(8, 8, dtype=torch.bfloat16, device="cuda")
        A = torch.zeros(E, 8, 8, device="cuda")
        B = torch.zeros(E, 8, 8, device="cuda")
        ctx = L.create_from_tensors([(W, A, B)], [(0, 0, 8, 8)], E, 8)
        cases = [rng.normal(0, 1, E).astype(np.float32) for _ in range(6)]
        tie = np.zeros(E, np.float32); tie[: min(E, 3)] = 1.0
        cases += [tie, np.full(E, -2.5, np.float32), np.where(np.arange(E) % 2 == 0, 0.0, -0.0).astype(np.float32),
                  (rng.integers(-2, 3, E)).astype(np.float32), np.linspace(80, -80, E).astype(np.float32)]
        ids_d = torch.full((8,), -7, dtype=torch.int32, device="cuda")
        gates_d = torch.full((8,), -7.0, dtype=torch.float32, device="cuda")
        for logits in cases:
            ld = torch.from_numpy(logits).cuda()
            L.lsw_route_dev(ctx, ld.data_ptr(), k, ids_d.data_ptr(), gates_d.data_ptr(), _stream())
            want_ids, want_gates = O.route(logits, k)
            got_ids, got_gates = ids_d.cpu().numpy()[:k], gates_d.cpu().numpy()[:k]
            assert got_ids.tolist() == want_ids.tolist(), (E, k, logits[:8])
            assert (_f32_ulp_distance(got_gates, want_gates) <= 1).all(), (E, k, got_gates, want_gates)
            assert abs(float(got_gates.astype(np.float64).sum()) - 1.0) < 1e-6
        assert L.lsw_dev_status(ctx) == 0
        bad = cases[0].copy(); bad[E // 2] = np.nan
        L.lsw_route_dev(ctx, torch.from_numpy(bad).cuda().data_ptr(), k, ids_d.data_ptr(), gates_d.data_ptr(), _stream())
        torch.cuda.synchronize()
        assert L.lsw_dev_status(ctx) & 1
        assert (ids_d.cpu().numpy()[:k] == -1).all()
        with pytest.raises(L.LswError):
            L.lsw_route_dev(ctx, ld.data_ptr(), 9, ids_d.data_ptr(), gates_d.data_ptr(), _stream())
        torch.cuda.synchronize()
        L.lsw_destroy(ctx)


@pytest.mark.parametrize("kernel", [L.KERNEL_VALU, L.KERNEL_MFMA])
def test_switch_dev_leaves_the_bits_of_the_host_driven_switch_and_matches_the_oracle(kernel):
    wl, host, dev_stack = _tiny_stack(kernel)
    _, _, host_stack = _tiny_stack(kernel)
    (W0, A, B), = host
    logits = I.router_logits(wl)
    logits[5] = logits[4]                       # a step that keeps both experts: the lists cancel, nothing is launched
    logits[7, :] = logits[6, :]
    logits[7, [0, 1]] = logits[7, [1, 0]]       # and steps that share experts
    bufs = [(torch.zeros(2, dtype=torch.int32, device="cuda"), torch.zeros(2, dtype=torch.float32, device="cuda")) for _ in range(2)]
    logits_d = torch.from_numpy(logits).cuda()
    prev = dev_stack.rows(0)
    old_host = NONE
    for t in range(len(logits)):
        new_d, old_d = bufs[t % 2], bufs[(t + 1) % 2]
        L.lsw_route_dev(dev_stack.ctx, logits_d[t].data_ptr(), wl.top_k, new_d[0].data_ptr(), new_d[1].data_ptr(), _stream())
        L.lsw_switch_dev(dev_stack.ctx, old_d[0].data_ptr(), old_d[1].data_ptr(), 0 if t == 0 else wl.top_k,
                         new_d[0].data_ptr(), new_d[1].data_ptr(), wl.top_k, stream=_stream())
        new_host = (new_d[0].cpu().numpy().copy(), new_d[1].cpu().numpy().copy())     # what the device routed
        assert new_host[0].tolist() == O.route(logits[t], wl.top_k)[0].tolist()
        host_stack.switch(old_host, new_host)
        got = dev_stack.rows(0)
        assert (got == host_stack.rows(0)).all(), t
        rep, _ = check_step(prev, got, A, B, old_host, new_host)
        assert rep["fail"] == 0, (t, {k: v for k, v in rep.items() if k != "fail_mask"})
        prev, old_host = got, new_host
    assert L.lsw_dev_status(dev_stack.ctx) == 0
    # the context no longer knows what is merged
    with pytest.raises(L.LswError) as e:
        L.lsw_get_state(dev_stack.ctx, 0)
    assert e.value.status == L.LSW_ERR_STATE
    L.lsw_set_option(dev_stack.ctx, L.LSW_OPT_STRICT_STATE, 1)
    with pytest.raises(L.LswError) as e:
        L.lsw_switch_dev(dev_stack.ctx, bufs[0][0].data_ptr(), bufs[0][1].data_ptr(), 2, bufs[1][0].data_ptr(), bufs[1][1].data_ptr(), 2, stream=_stream())
    assert e.value.status == L.LSW_ERR_STATE
    dev_stack.close()
    host_stack.close()


def test_switch_dev_refuses_bad_lists_without_touching_a_weight():
    wl, host, ds = _tiny_stack()
    W = ds.stack[0][0]
    W.view(torch.int16)[0, :4] = torch.tensor([-32768, 0, -32768, 0], dtype=torch.int16, device="cuda")   # -0, +0: any launch would turn -0 into +0
    before = ds.rows(0)
    good = _dev_lists([1, 2], [0.25, 0.75])
    for bad_ids, bad_gates, k in [([3, 3], [0.5, 0.5], 2), ([1, 8], [0.5, 0.5], 2), ([-1, 2], [0.5, 0.5], 2),
                                  ([1, 2], [np.nan, 0.5], 2), ([1, 2], [np.inf, 0.5], 2)]:
        bad = _dev_lists(bad_ids, bad_gates)
        for old, new in [(good, bad), (bad, good)]:
            L.lsw_switch_dev(ds.ctx, old[0].data_ptr(), old[1].data_ptr(), 2, new[0].data_ptr(), new[1].data_ptr(), k, stream=_stream())
            torch.cuda.synchronize()
            assert (ds.rows(0) == before).all(), (bad_ids, bad_gates)
    assert L.lsw_dev_status(ds.ctx) & 2
    # identical lists cancel completely: nothing may change either, the -0 included
    L.lsw_switch_dev(ds.ctx, good[0].data_ptr(), good[1].data_ptr(), 2, good[0].data_ptr(), good[1].data_ptr(), 2, stream=_stream())
    torch.cuda.synchronize()
    assert (ds.rows(0) == before).all()
    # what the host can check it checks: nothing launched, status returned
    for args in [dict(k_old=9), dict(k_new=-1), dict(old_ids=0)]:
        with pytest.raises(L.LswError) as e:
            L.lsw_switch_dev(ds.ctx, args.get("old_ids", good[0].data_ptr()), good[1].data_ptr(), args.get("k_old", 2),
                             good[0].data_ptr(), good[1].data_ptr(), args.get("k_new", 2), stream=_stream())
        assert e.value.status == L.LSW_ERR_ARG
    assert (ds.rows(0) == before).all()
    ds.close()


def test_router_logits_gemv_then_route_then_switch_then_decode_recorded_in_a_graph():
    """A whole token step (router GEMV, device router, device switch, merged decode) recorded in HIP graphs (one per
    parity of the ping-pong list buffers) and replayed with fresh inputs, with eager work and synchronisations between
    the replays; every replay is compared bit for bit with the same step issued eagerly on a twin stack, and with the
    oracle applied to the state before it."""
    wl = I.Workload("mini", 2, 64, 136, 32, 8, 8, 2, 4, 0.02, 1 / 8, 0.01, 616)
    host = I.host_stack(wl)
    twins = [DeviceStack.from_host(host, wl.linear_shapes(), wl.experts, wl.rank) for _ in range(2)]
    rng = np.random.default_rng(3)
    hidden = 64
    Wg = torch.from_numpy(I.f32_to_bf16_bits(rng.normal(0, 0.5, (wl.experts, hidden)).astype(np.float32)).view(np.int16)).cuda().view(torch.bfloat16)
    nx = L.lsw_query(twins[0].ctx, L.LSW_Q_GEMV_X_ELEMS)
    ny = L.lsw_query(twins[0].ctx, L.LSW_Q_GEMV_Y_ELEMS)
    x_router = torch.zeros(hidden, dtype=torch.bfloat16, device="cuda")       # the token's router input (first layer's input)
    xall = torch.randn(nx, device="cuda").to(torch.bfloat16)

    class State:
        def __init__(self, ds):
            self.ds = ds
            self.logits = torch.zeros(wl.experts, device="cuda")
            self.bufs = [(torch.zeros(2, dtype=torch.int32, device="cuda"), torch.zeros(2, dtype=torch.float32, device="cuda")) for _ in range(2)]
            self.y = torch.zeros(ny, device="cuda")
            first = _dev_lists([0, 1], [0.5, 0.5])
            self.bufs[1][0].copy_(first[0]); self.bufs[1][1].copy_(first[1])
            L.lsw_switch_dev(ds.ctx, 0, 0, 0, self.bufs[1][0].data_ptr(), self.bufs[1][1].data_ptr(), 2, stream=_stream())

        def token(self, parity, stream):
            new, old = self.bufs[parity], self.bufs[1 - parity]
            L.lsw_gemv_bf16(Wg.data_ptr(), x_router.data_ptr(), self.logits.data_ptr(), wl.experts, hidden, stream)
            L.lsw_route_dev(self.ds.ctx, self.logits.data_ptr(), 2, new[0].data_ptr(), new[1].data_ptr(), stream)
            L.lsw_switch_dev(self.ds.ctx, old[0].data_ptr(), old[1].data_ptr(), 2, new[0].data_ptr(), new[1].data_ptr(), 2, stream=stream)
            L.lsw_merged_gemv_all(self.ds.ctx, xall.data_ptr(), self.y.data_ptr(), stream)

    eager, graphed = State(twins[0]), State(twins[1])
    # both twins take two eager tokens first: launch plans and kernel attributes are set up on first use, which must
    # not happen while recording
    for parity in (0, 1):
        x_router.copy_(torch.randn(hidden, device="cuda").to(torch.bfloat16))
        eager.token(parity, _stream())
        graphed.token(parity, _stream())
    torch.cuda.synchronize()
    graphs = []
    for parity in (0, 1):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            graphed.token(parity, _stream())       # recorded, not run
        graphs.append(g)
    torch.cuda.synchronize()
    for p in range(len(host)):
        assert (twins[0].rows(p) == twins[1].rows(p)).all()
    for t in range(8):
        parity = t % 2
        x_router.copy_(torch.randn(hidden, device="cuda").to(torch.bfloat16))      # eager work between the replays
        before = [twins[1].rows(p) for p in range(len(host))]
        old = (graphed.bufs[1 - parity][0].cpu().numpy().copy(), graphed.bufs[1 - parity][1].cpu().numpy().copy())
        eager.token(parity, _stream())
        graphs[parity].replay()
        torch.cuda.synchronize()
        assert torch.equal(eager.logits, graphed.logits) and torch.equal(eager.y, graphed.y)
        new = (graphed.bufs[parity][0].cpu().numpy().copy(), graphed.bufs[parity][1].cpu().numpy().copy())
        assert torch.equal(eager.bufs[parity][0], graphed.bufs[parity][0]) and torch.equal(eager.bufs[parity][1], graphed.bufs[parity][1])
        want_ids, want_gates = O.route(graphed.logits.cpu().numpy(), 2)
        assert new[0].tolist() == want_ids.tolist()
        assert (_f32_ulp_distance(new[1], want_gates) <= 1).all()
        # the router's logits themselves: W_g x in fp64
        lg = O.gemv(Wg.view(torch.int16).cpu().numpy().view(np.uint16), x_router.view(torch.int16).cpu().numpy().view(np.uint16))
        assert np.allclose(graphed.logits.cpu().numpy(), lg, rtol=0, atol=1e-4)
        for p, (W, A, B) in enumerate(host):
            got = twins[1].rows(p)
            assert (twins[0].rows(p) == got).all(), (t, p)
            rep, _ = check_step(before[p], got, A, B, old, new)
            assert rep["fail"] == 0, (t, p, {k: v for k, v in rep.items() if k != "fail_mask"})
    assert L.lsw_dev_status(twins[0].ctx) == 0 and L.lsw_dev_status(twins[1].ctx) == 0
    for ds in twins:
        ds.close()
