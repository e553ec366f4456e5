"""The hot path under HIP graph capture.  The attention-sized calls (Section 7.4: many small matrix products)
are launch-bound, so a caller will want to capture them; the library only enqueues kernels on the caller's
stream (no allocation, no synchronisation, no memset), which is what capture needs.  The captured step is
replayed several times with eager work and synchronisations in between, and every replay is compared with
the eager result and with the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2402_02320_amd import spin, workloads

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).cuda()


def host(t):
    return t.cpu().numpy().view(np.uint64)


@pytest.mark.parametrize("path", [spin.LIMB_MFMA, spin.VALU])
def test_captured_attention_step_replays_bit_exact(path):
    c = workloads.CONFIGS[4]
    n, f = c.n, c.f
    Q, KT = workloads.gemm_plaintexts(4, 0)                     # [64,128,64], [64,64,128]
    batch, M, K = Q.shape
    N = KT.shape[2]
    xe, ye = oracle.encode(Q, f), oracle.encode(KT, f)
    A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=c.seed)
    count = batch * M * N
    r, rt, rm = oracle.trunc_dealer(n, count, f, seed=c.seed)
    ea, eb, ec = oracle.dealer_mul(n, count, seed=c.seed + 1)
    w = oracle.share(oracle.encode(workloads.vec_plaintexts(4)[0], f), n, c.seed, 9)

    x, y = dev(xe), dev(ye)
    Ad, Bd, Cd, rd, rtd, rmd = (dev(t) for t in (A, B, C, r, rt, rm))
    ead, ebd, ecd, wd = (dev(t) for t in (ea, eb, ec, w))
    Xs = torch.empty((n, batch, M, K), dtype=torch.int64, device="cuda")
    Ys = torch.empty((n, batch, K, N), dtype=torch.int64, device="cuda")
    Z = torch.empty((n, batch, M, N), dtype=torch.int64, device="cuda")
    T = torch.empty((n, count), dtype=torch.int64, device="cuda")
    V = torch.empty((n, count), dtype=torch.int64, device="cuda")
    ws = torch.empty(spin.beaver_matmul_workspace_bytes(n, batch, M, N, K, path), dtype=torch.uint8, device="cuda")

    def step():
        spin.share(x, n, c.seed, oracle.STREAM_X, out=Xs)
        spin.share(y, n, c.seed, oracle.STREAM_Y, out=Ys)
        spin.beaver_matmul(Xs, Ys, Ad, Bd, Cd, path=path, out=Z, workspace=ws)
        spin.trunc(Z.view(n, -1), rd, rtd, rmd, f, out=T)
        spin.beaver_mul(T, wd, ead, ebd, ecd, out=V)

    step()                                                      # eager: also sets the kernel attributes
    torch.cuda.synchronize()
    eager_T, eager_V = T.clone(), V.clone()
    # the oracle's view of the same step
    X, Y = oracle.share(xe, n, c.seed, oracle.STREAM_X), oracle.share(ye, n, c.seed, oracle.STREAM_Y)
    To = oracle.trunc(oracle.beaver_matmul(X, Y, A, B, C).reshape(n, -1), r, rt, rm, f)
    assert (host(eager_T) == To).all()
    assert (host(eager_V) == oracle.beaver_mul(To, w, ea, eb, ec)).all()

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for replay in range(4):
        for t in (Xs, Ys, Z, T, V):
            t.fill_(replay + 1)                                 # eager work between replays; stale outputs destroyed
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(T, eager_T), replay
        assert torch.equal(V, eager_V), replay
