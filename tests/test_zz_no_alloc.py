"""lsw_adapter_forward_static (the entry point that allocates nothing: its workspace is a device array inside the
library) against lsw_adapter_forward with a caller-supplied workspace, through the C ABI.

The two run the same kernels, so the outputs must be identical bit for bit, which is inside the bar the prompt path is
held to against the oracle (tests/test_gpu_adapter_path.py); the first call's output is also checked against the oracle
itself.  Two calls in a row share the array, the second with a smaller input; sizes beyond the array are refused before
anything is launched."""
import numpy as np
import pytest
import torch

from oracle import compare as C
from oracle import lsw_oracle as O
from paper_2405_17741_amd import binding as L
from paper_2405_17741_amd import inputs as I
from tests.gpu_harness import DeviceStack, bits_to_device, device_to_bits

pytestmark = pytest.mark.gpu


def _tokens(rng, T, E, k, inn, out):
    X = I.f32_to_bf16_bits(rng.normal(0, 1, (T, inn)).astype(np.float32))
    Y = I.f32_to_bf16_bits(rng.normal(0, 0.5, (T, out)).astype(np.float32))
    routes = [O.route(l, k) for l in rng.normal(0, 1, (T, E)).astype(np.float32)]
    ids = np.stack([r[0] for r in routes]).astype(np.int32).reshape(T, k)
    gates = np.stack([r[1] for r in routes]).astype(np.float32).reshape(T, k)
    return X, Y, ids, gates


def _both(ds, p, X, Y, ids, gates, k):
    """(output of the static entry point, output of the one with a caller's workspace) on the same inputs."""
    T = X.shape[0]
    stream = torch.cuda.current_stream().cuda_stream
    Xd = bits_to_device(X)
    idd, gd = torch.from_numpy(ids).cuda(), torch.from_numpy(gates).cuda()
    Ya, Yb = bits_to_device(Y), bits_to_device(Y)
    ws = torch.full((L.lsw_adapter_workspace_bytes(ds.ctx, p, T) // 4 + 64,), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    L.lsw_adapter_forward_static(ds.ctx, p, Xd.data_ptr(), T, idd.data_ptr(), gd.data_ptr(), k, Ya.data_ptr(), stream)
    free_after, _ = torch.cuda.mem_get_info()
    assert free_after >= free_before           # the device's free memory did not shrink: nothing was allocated
    L.lsw_adapter_forward(ds.ctx, p, Xd.data_ptr(), T, idd.data_ptr(), gd.data_ptr(), k, Yb.data_ptr(), ws.data_ptr(), stream)
    torch.cuda.synchronize()
    return device_to_bits(Ya), device_to_bits(Yb)


def test_static_workspace_entry_point_equals_the_one_with_a_callers_workspace():
    E, r, k = 8, 8, 2
    shapes = [(0, 0, 264, 520), (0, 1, 136, 1032)]            # two linears: the second call also changes the linear
    rng = np.random.default_rng(2024)
    host = [I.host_linear(rng, o, n, E, r, 0.02, 1 / np.sqrt(n), 0.05) for _, _, o, n in shapes]
    ds = DeviceStack.from_host(host, shapes, E, r, scale=0.5)
    with pytest.raises(L.LswError) as e:                       # before the path is enabled
        L.lsw_adapter_forward_static(ds.ctx, 0, 16, 1, 16, 16, 1, 16)
    assert e.value.status == L.LSW_ERR_STATE
    L.lsw_enable_adapter_path(ds.ctx)

    # first call: 700 tokens through linear 0
    X, Y, ids, gates = _tokens(rng, 700, E, k, 520, 264)
    got_static, got_ws = _both(ds, 0, X, Y, ids, gates, k)
    assert (got_static == got_ws).all()
    (_, A, B) = host[0]
    rep = C.switch_parity(got_static, O.adapter_forward(Y, X, A, B, ids, gates, 0.5), Y, O.adapter_magnitude(X, A, B, ids, gates, 0.5))
    assert rep["fail"] == 0 and rep["exact"] > 0.995 * rep["n"]
    assert (got_static != Y).mean() > 0.2

    # second call right behind it, smaller: 45 tokens through linear 1 (the array still holds the first call's sums)
    X2, Y2, ids2, gates2 = _tokens(rng, 45, E, k, 1032, 136)
    got_static2, got_ws2 = _both(ds, 1, X2, Y2, ids2, gates2, k)
    assert (got_static2 == got_ws2).all()
    (_, A1, B1) = host[1]
    rep = C.switch_parity(got_static2, O.adapter_forward(Y2, X2, A1, B1, ids2, gates2, 0.5), Y2, O.adapter_magnitude(X2, A1, B1, ids2, gates2, 0.5))
    assert rep["fail"] == 0

    # and the first one again: nothing of the smaller call is left in the way
    got_static3, _ = _both(ds, 0, X, Y, ids, gates, k)
    assert (got_static3 == got_static).all()
    assert L.lsw_dev_status(ds.ctx) == 0

    # beyond the array: refused with a clear error, nothing launched (Y unchanged)
    T_big = 1
    while L.lsw_adapter_workspace_bytes(ds.ctx, 0, T_big) <= 32 << 20:
        T_big *= 2
    Yd = bits_to_device(Y)
    with pytest.raises(L.LswError) as e:
        L.lsw_adapter_forward_static(ds.ctx, 0, 16, T_big, 16, 16, k, Yd.data_ptr())
    assert e.value.status == L.LSW_ERR_SHAPE and "workspace" in str(e.value)
    torch.cuda.synchronize()
    assert (device_to_bits(Yd) == Y).all()
    ds.close()


def test_a_second_context_on_the_same_gpu_shares_the_array():
    E, r, k = 4, 16, 2
    rng = np.random.default_rng(7)
    outs = []
    for _ in range(2):                                         # two contexts, one after the other, same inputs
        rng_c = np.random.default_rng(99)
        host = [I.host_linear(rng_c, 72, 264, E, r, 0.02, 1 / 16, 0.05)]
        ds = DeviceStack.from_host(host, [(0, 0, 72, 264)], E, r)
        L.lsw_enable_adapter_path(ds.ctx)
        X, Y, ids, gates = _tokens(np.random.default_rng(5), 130, E, k, 264, 72)
        a, b = _both(ds, 0, X, Y, ids, gates, k)
        assert (a == b).all()
        outs.append(a)
        ds.close()
    assert (outs[0] == outs[1]).all()
