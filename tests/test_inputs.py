"""Checks of the synthetic input recipe (shapes, sizes, distributions, reuse statistics)."""
import numpy as np

from paper_2405_17741_amd import inputs as I


def test_workload_sizes_match_the_stated_workloads():
    assert I.WORKLOADS["tiny"].w_elements() == 65536
    assert I.WORKLOADS["7b"].w_elements() == 6_476_005_376
    assert I.WORKLOADS["7b_r64"].w_elements() == 6_476_005_376
    assert I.WORKLOADS["13b"].w_elements() == 12_687_769_600
    assert I.WORKLOADS["70b"].w_elements() == 68_451_041_280
    wl = I.WORKLOADS["7b"]
    shapes = wl.linear_shapes()
    assert len(shapes) == 224
    assert [(o, i) for _, _, o, i in shapes[:7]] == [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)]
    s70 = I.WORKLOADS["70b"].linear_shapes()[:7]
    assert [(o, i) for _, _, o, i in s70] == [(8192, 8192), (1024, 8192), (1024, 8192), (8192, 8192),
                                             (28672, 8192), (28672, 8192), (8192, 28672)]


def test_host_stack_is_seeded_and_distributed_as_stated():
    wl = I.WORKLOADS["tiny"]
    (W, A, B), = I.host_stack(wl)
    (W2, A2, B2), = I.host_stack(wl)
    assert (W == W2).all() and (A == A2).all() and (B == B2).all()
    assert W.shape == (256, 256) and W.dtype == np.uint16
    assert A.shape == (8, 8, 256) and B.shape == (8, 256, 8) and A.dtype == np.float32
    w = (W.astype(np.uint32) << 16).view(np.float32)
    assert abs(w.std() - 0.02) < 0.001 and abs(A.std() - 1 / 16) < 0.002 and abs(B.std() - 0.01) < 0.0005
    assert abs(w.mean()) < 3e-4


def test_router_logit_stream_reuse_statistics():
    # i.i.d. N(0,1) logits, E=8, top-2: P(consecutive sets share >= 1 expert) = 1 - C(6,2)/C(8,2) = 13/28
    wl = I.Workload("s", 1, 8, 8, 8, 8, 8, 2, 0, 0.02, 0.1, 0.01, 77)
    L = I.router_logits(wl, steps=20000)
    top = np.argsort(-L, axis=1, kind="stable")[:, :2]
    share = np.array([len(set(top[t]) & set(top[t - 1])) > 0 for t in range(1, len(top))])
    assert abs(share.mean() - 13 / 28) < 0.012
    # E=16: 1 - C(14,2)/C(16,2) = 29/120
    wl16 = I.Workload("s", 1, 8, 8, 8, 16, 8, 2, 0, 0.02, 0.1, 0.01, 78)
    L = I.router_logits(wl16, steps=20000)
    top = np.argsort(-L, axis=1, kind="stable")[:, :2]
    share = np.array([len(set(top[t]) & set(top[t - 1])) > 0 for t in range(1, len(top))])
    assert abs(share.mean() - 29 / 120) < 0.012
    # forced reuse: P = 1 - (1 - 29/120) * (1 - 0.5)
    wlf = I.Workload("s", 1, 8, 8, 8, 16, 8, 2, 0, 0.02, 0.1, 0.01, 79, reuse_prob=0.5)
    L = I.router_logits(wlf, steps=20000)
    top = np.argsort(-L, axis=1, kind="stable")[:, :2]
    share = np.array([len(set(top[t]) & set(top[t - 1])) > 0 for t in range(1, len(top))])
    assert abs(share.mean() - (1 - (91 / 120) * 0.5)) < 0.012
    assert abs(L.std() - 1.0) < 0.02


def test_sample_rows():
    rng = np.random.default_rng(0)
    r = I.sample_rows(rng, 4096)
    assert r[0] == 0 and r[1] == 1 and r[-1] == 4095 and len(set(r.tolist())) == len(r) and 61 <= len(r) <= 64
    assert I.sample_rows(rng, 2).tolist() == [0, 1]
