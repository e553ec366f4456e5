"""Attention-shaped composition of the two hot-path calls (Sections 7.3 and 7.4): the last Softmax
multiplication E * R folded into V, (E * R) @ V = E @ (R * V), with the matrix products batched over
heads.  Shapes: LeViT-256's D1 = D2 = 196, D3 = 64 and the original attention's 512 / 64.  Every GPU
call is compared bit for bit with the oracle; the ring identity is checked without the intermediate
truncations and the decoded results of both orders against float64."""
import numpy as np
import pytest
import torch

import oracle
from paper_2402_02320_amd import spin

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).cuda()


def host(t):
    return t.cpu().numpy().view(np.uint64)


def shared(x, n, f, seed, stream):
    return oracle.share(oracle.encode(x, f), n, seed, stream)


def mul_both(x, y, n, seed):
    """Elementwise Beaver mul on GPU and oracle; asserts equality, returns (gpu tensor, oracle array)."""
    count = x[0].size
    a, b, c = oracle.dealer_mul(n, count, seed=seed)
    zo = oracle.beaver_mul(x.reshape(n, -1), y.reshape(n, -1), a, b, c)
    zd = spin.beaver_mul(dev(x.reshape(n, -1)), dev(y.reshape(n, -1)), dev(a), dev(b), dev(c))
    assert (host(zd) == zo).all()
    return zd, zo


def trunc_both(zd, zo, n, f, seed):
    r, rt, rm = oracle.trunc_dealer(n, zo[0].size, f, seed=seed)
    to = oracle.trunc(zo.reshape(n, -1), r, rt, rm, f)
    td = spin.trunc(zd.view(n, -1), dev(r), dev(rt), dev(rm), f)
    assert (host(td) == to).all()
    return td, to


def matmul_both(X, Y, n, seed, path):
    _, batch, M, K = X.shape
    N = Y.shape[3]
    A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=seed)
    zo = oracle.beaver_matmul(X, Y, A, B, C)
    zd = spin.beaver_matmul(dev(X), dev(Y), dev(A), dev(B), dev(C), path=path)
    assert (host(zd) == zo).all()
    return zd, zo


@pytest.mark.parametrize("n,heads,D1,D3", [(3, 4, 196, 64), (2, 2, 512, 64)])
@pytest.mark.parametrize("path", [pytest.param(spin.LIMB_MFMA, id="limb"), pytest.param(spin.VALU, id="valu")])
def test_downsized_batch_multiplication(n, heads, D1, D3, path):
    f, D2 = 14, D1                                       # the paper runs attention at precision 14 (Section 7.2)
    rng = np.random.default_rng(D1 + n)
    scores = rng.normal(0, 1, size=(heads, D1, D2))
    E = np.exp(scores - scores.max(axis=1, keepdims=True))          # Softmax numerators, in (0, 1]
    R = (1.0 / E.sum(axis=1))[:, :, None]                           # reciprocal of the column sums: 1 x D2 per head
    V = rng.normal(0, 1, size=(heads, D2, D3))
    want = np.matmul(E * R.transpose(0, 2, 1), V)
    seed = 0xA77
    Es, Vs = shared(E, n, f, seed, 1), shared(V, n, f, seed, 2)
    Rrow = shared(np.broadcast_to(R.transpose(0, 2, 1), E.shape).copy(), n, f, seed, 3)   # R tiled D1 times
    Rcol = shared(np.broadcast_to(R, V.shape).copy(), n, f, seed, 3)                      # R tiled D3 times

    # naive order: Mul on D1 x D2 elements, then MatMul
    sd, so = mul_both(Es, Rrow, n, seed + 1)
    std, sto = trunc_both(sd, so, n, f, seed + 2)
    od, oo = matmul_both(sto.reshape(Es.shape), Vs, n, seed + 3, path)
    otd, _ = trunc_both(od, oo, n, f, seed + 4)
    naive = oracle.decode(host(spin.open(otd)), f).reshape(want.shape)

    # downsized order: Mul on D2 x D3 elements, then MatMul
    wd, wo = mul_both(Rcol, Vs, n, seed + 5)
    wtd, wto = trunc_both(wd, wo, n, f, seed + 6)
    pd, po = matmul_both(Es, wto.reshape(Vs.shape), n, seed + 7, path)
    ptd, _ = trunc_both(pd, po, n, f, seed + 8)
    down = oracle.decode(host(spin.open(ptd)), f).reshape(want.shape)

    bound = 2.0 ** -f * (D2 + 2) * 2
    assert np.abs(naive - want).max() <= bound
    assert np.abs(down - want).max() <= bound

    # the identity itself, exact in the ring when the intermediate truncations are left out (precision 3f)
    lhs = matmul_both(so.reshape(Es.shape), Vs, n, seed + 9, path)[1]
    rhs = matmul_both(Es, wo.reshape(Vs.shape), n, seed + 10, path)[1]
    assert (oracle.open_(lhs) == oracle.open_(rhs)).all()
    assert np.abs(oracle.decode(oracle.open_(lhs), 3 * f) - want).max() <= 2.0 ** -f * (D2 + 2) * 2
    # and the sizes the paper quotes: the elementwise product shrinks by D1 / D3
    assert so[0].size // wo[0].size == D1 // D3


@pytest.mark.parametrize("n,outer,mid,inner", [(1, 1, 1, 1), (2, 1, 7, 1), (3, 2, 5, 33), (5, 4, 196, 64), (2, 3, 100, 257),
                                               (8, 1, 3, 1000)])
@pytest.mark.parametrize("over_inner", [True, False])
def test_tiled_factor_multiplication_matches_the_oracle(n, outer, mid, inner, over_inner):
    rng = np.random.default_rng(n * 100 + mid + inner)
    small = outer * (mid if over_inner else inner)
    x = rng.integers(0, 1 << 64, size=small, dtype=np.uint64)
    y = rng.integers(0, 1 << 64, size=outer * mid * inner, dtype=np.uint64)
    X, Y = oracle.share(x, n, 5, oracle.STREAM_X), oracle.share(y, n, 5, oracle.STREAM_Y)
    a, b, c = oracle.dealer_mul_bcast(n, outer, mid, inner, over_inner, seed=6)
    want = oracle.beaver_mul_bcast(X, Y, a, b, c, outer, mid, inner, over_inner)
    full = (n, outer, mid, inner)
    sshape = (n, outer, mid) if over_inner else (n, outer, inner)
    yd = dev(Y.reshape(full))
    got = spin.beaver_mul_bcast(dev(X.reshape(sshape)), yd, dev(a.reshape(sshape)), dev(b.reshape(full)),
                                dev(c.reshape(full)), over_inner)
    assert (host(got).reshape(n, -1) == want).all()
    # in place on the large operand
    spin.beaver_mul_bcast(dev(X.reshape(sshape)), yd, dev(a.reshape(sshape)), dev(b.reshape(full)),
                          dev(c.reshape(full)), over_inner, out=yd)
    assert (host(yd).reshape(n, -1) == want).all()


def test_tiled_factor_multiplication_at_streaming_size():
    n, outer, mid, inner = 3, 8, 512, 1024                      # 3 x 4 Mi words: past the non-temporal threshold
    rng = np.random.default_rng(9)
    for over_inner in (True, False):
        small = outer * (mid if over_inner else inner)
        x = rng.integers(0, 1 << 64, size=small, dtype=np.uint64)
        y = rng.integers(0, 1 << 64, size=outer * mid * inner, dtype=np.uint64)
        X, Y = oracle.share(x, n, 5, oracle.STREAM_X), oracle.share(y, n, 5, oracle.STREAM_Y)
        a, b, c = oracle.dealer_mul_bcast(n, outer, mid, inner, over_inner, seed=6)
        want = oracle.beaver_mul_bcast(X, Y, a, b, c, outer, mid, inner, over_inner)
        full = (n, outer, mid, inner)
        sshape = (n, outer, mid) if over_inner else (n, outer, inner)
        got = spin.beaver_mul_bcast(dev(X.reshape(sshape)), dev(Y.reshape(full)), dev(a.reshape(sshape)),
                                    dev(b.reshape(full)), dev(c.reshape(full)), over_inner)
        assert (host(got).reshape(n, -1) == want).all()


def test_downsized_order_with_the_factor_tiled_inside_the_kernel():
    # E @ (R * V) with R [1 x D2] handed over untiled: R scales the rows of V
    n, heads, D2, D3, f = 3, 4, 196, 64, 14
    rng = np.random.default_rng(11)
    Rr = rng.uniform(0.001, 0.05, size=(heads, D2))
    V = rng.normal(0, 1, size=(heads, D2, D3))
    Rs, Vs = shared(Rr, n, f, 21, 1), shared(V, n, f, 21, 2)
    a, b, c = oracle.dealer_mul_bcast(n, heads, D2, D3, True, seed=22)
    wo = oracle.beaver_mul_bcast(Rs.reshape(n, -1), Vs.reshape(n, -1), a, b, c, heads, D2, D3, True)
    wd = spin.beaver_mul_bcast(dev(Rs), dev(Vs), dev(a.reshape(n, heads, D2)), dev(b.reshape(Vs.shape)),
                               dev(c.reshape(Vs.shape)), True)
    assert (host(wd).reshape(n, -1) == wo).all()
    wtd, wto = trunc_both(wd.view(n, -1), wo, n, f, 23)
    got = oracle.decode(host(spin.open(wtd)), f).reshape(V.shape)
    assert np.abs(got - Rr[:, :, None] * V).max() <= 2.0 ** -f * 3 * max(1.0, np.abs(V).max())


@pytest.mark.parametrize("path", [pytest.param(spin.LIMB_MFMA, id="limb"), pytest.param(spin.VALU, id="valu")])
def test_grouped_matmuls_of_different_shapes_in_one_call(path):
    # the attention products of three LeViT-like stages (196, 49 and 16 tokens) in one call: Q.K^T with K
    # stored untransposed, then P.V; plus products that take the tile kernel (long inner dimension, many column
    # tiles), an odd inner dimension and a 1 x 1 x 1 product.  Every group against the oracle, and against the
    # same products submitted one call at a time (on the limb path the grouped call shares launches).
    n = 3
    rng = np.random.default_rng(77)
    shapes = [(4, 196, 196, 64, True), (4, 196, 64, 196, False), (8, 49, 49, 32, True), (8, 49, 32, 49, False),
              (12, 16, 16, 32, True), (1, 1, 1, 1, False), (1, 130, 200, 1030, False), (2, 70, 150, 999, True),
              (1, 300, 64, 40, False)]
    groups, wants = [], []
    for idx, (batch, M, N, K, yt) in enumerate(shapes):
        X = rng.integers(0, 1 << 64, size=(n, batch, M, K), dtype=np.uint64)
        Y = rng.integers(0, 1 << 64, size=(n, batch, K, N), dtype=np.uint64)
        A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=700 + idx)
        wants.append(oracle.beaver_matmul(X, Y, A, B, C))
        if yt:
            Y, B = np.ascontiguousarray(Y.transpose(0, 1, 3, 2)), np.ascontiguousarray(B.transpose(0, 1, 3, 2))
        groups.append({"X": dev(X), "Y": dev(Y), "A": dev(A), "B": dev(B), "C": dev(C), "y_transposed": yt})
    outs = spin.beaver_matmul_grouped(groups, path=path)
    for z, want, g in zip(outs, wants, groups):
        assert (host(z) == want).all()
        single = spin.beaver_matmul(g["X"], g["Y"], g["A"], g["B"], g["C"], path=path, y_transposed=g["y_transposed"])
        assert torch.equal(z, single)
    # in place on C, and a second call on the same workspace
    ws = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
    for g in groups:
        g["out"] = g["C"]
    spin.beaver_matmul_grouped(groups, path=path, workspace=ws)
    for g, want in zip(groups, wants):
        assert (host(g["C"]) == want).all()


def test_more_groups_than_one_launch_table_holds():
    # 40 groups of five different shapes and 2 parties: the descriptor tables are sent 32 groups at a time
    n = 2
    rng = np.random.default_rng(78)
    base = [(1, 33, 70, 34, False), (2, 64, 64, 64, True), (1, 100, 31, 96, False), (3, 17, 130, 20, True), (1, 128, 128, 250, False)]
    groups, wants = [], []
    for idx in range(40):
        batch, M, N, K, yt = base[idx % 5]
        M += idx // 5
        X = rng.integers(0, 1 << 64, size=(n, batch, M, K), dtype=np.uint64)
        Y = rng.integers(0, 1 << 64, size=(n, batch, K, N), dtype=np.uint64)
        A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=900 + idx)
        wants.append(oracle.beaver_matmul(X, Y, A, B, C))
        if yt:
            Y, B = np.ascontiguousarray(Y.transpose(0, 1, 3, 2)), np.ascontiguousarray(B.transpose(0, 1, 3, 2))
        groups.append({"X": dev(X), "Y": dev(Y), "A": dev(A), "B": dev(B), "C": dev(C), "y_transposed": yt})
    for z, want in zip(spin.beaver_matmul_grouped(groups), wants):
        assert (host(z) == want).all()


def test_grouped_call_with_five_parties_takes_the_tile_kernel_for_every_group():
    # more than three parties: no group is eligible for the row-streaming kernel, all left operands are packed
    n = 5
    rng = np.random.default_rng(79)
    shapes = [(2, 64, 64, 64, True), (1, 200, 64, 130, False), (3, 33, 129, 48, False), (1, 128, 256, 512, True)]
    groups, wants = [], []
    for idx, (batch, M, N, K, yt) in enumerate(shapes):
        X = rng.integers(0, 1 << 64, size=(n, batch, M, K), dtype=np.uint64)
        Y = rng.integers(0, 1 << 64, size=(n, batch, K, N), dtype=np.uint64)
        A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=950 + idx)
        wants.append(oracle.beaver_matmul(X, Y, A, B, C))
        if yt:
            Y, B = np.ascontiguousarray(Y.transpose(0, 1, 3, 2)), np.ascontiguousarray(B.transpose(0, 1, 3, 2))
        groups.append({"X": dev(X), "Y": dev(Y), "A": dev(A), "B": dev(B), "C": dev(C), "y_transposed": yt})
    for z, want in zip(spin.beaver_matmul_grouped(groups), wants):
        assert (host(z) == want).all()
