"""GPU-vs-oracle parity through the C ABI: every share bit-exact on the same
seeded inputs, at sizes that span several tiles and a ragged tail, on the edge
cases, and at the full size of every benchmark configuration (whole tensors:
every share word of the product and of the truncated product, the
reconstruction and the decoded bound over every row).  Inputs and expected
values come from oracle/ and the workload generators only."""
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


def rand_u64(rng, shape):
    return rng.integers(0, 1 << 64, size=shape, dtype=np.uint64)


# ----------------------------------------------------------------------------- generator / share / open
@pytest.mark.parametrize("count,first", [(1, 0), (2, 5), (255, 0), (256, 1 << 40), (1000, 3), (65537, 0)])
def test_random_matches_generator_spec(count, first):
    got = host(spin.random(count, seed=0xABC, stream_id=4, party=2, first_idx=first))
    assert (got == oracle.random(count, 0xABC, 4, 2, first)).all()


@pytest.mark.parametrize("n", [1, 2, 3, 5, 8])
@pytest.mark.parametrize("count", [1, 2, 513, 4096, 100003])
def test_share_and_open(n, count):
    rng = np.random.default_rng(count + n)
    x = rand_u64(rng, count)
    want = oracle.share(x, n, 77, oracle.STREAM_X)
    got = spin.share(dev(x), n, 77, oracle.STREAM_X)
    assert (host(got) == want).all()
    assert (host(spin.open(got)) == x).all()
    mask = rand_u64(rng, (n, count))
    assert (host(spin.open(got, dev(mask))) == oracle.open_(want, mask)).all()


# ----------------------------------------------------------------------------- elementwise Beaver mul / trunc
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("count", [1, 2, 777, 70000])
def test_beaver_mul(n, count):
    rng = np.random.default_rng(1000 * n + count)
    x, y = rand_u64(rng, (n, count)), rand_u64(rng, (n, count))
    a, b, c = oracle.dealer_mul(n, count, seed=5)
    want = oracle.beaver_mul(x, y, a, b, c)
    got = spin.beaver_mul(dev(x), dev(y), dev(a), dev(b), dev(c))
    assert (host(got) == want).all()
    # in place on x
    xd = dev(x)
    spin.beaver_mul(xd, dev(y), dev(a), dev(b), dev(c), out=xd)
    assert (host(xd) == want).all()


@pytest.mark.parametrize("n,f", [(1, 16), (2, 16), (3, 16), (5, 16), (8, 16), (3, 1), (2, 61), (5, 26)])
@pytest.mark.parametrize("count", [1, 2, 999, 65536 + 2])
def test_trunc(n, f, count):
    rng = np.random.default_rng(n * 100 + f + count)
    xs = rng.integers(-(1 << 62), 1 << 62, size=count, dtype=np.int64)
    xs[0] = -(1 << 62)
    X = oracle.share(xs.view(np.uint64), n, 91, oracle.STREAM_X)
    r, rt, rm = oracle.trunc_dealer(n, count, f, seed=91)
    want = oracle.trunc(X, r, rt, rm, f)
    Xd = dev(X)
    got = spin.trunc(Xd, dev(r), dev(rt), dev(rm), f)
    assert (host(got) == want).all()
    spin.trunc(Xd, dev(r), dev(rt), dev(rm), f, out=Xd)          # in place
    assert (host(Xd) == want).all()


@pytest.mark.parametrize("n,f", [(1, 16), (2, 16), (3, 14), (5, 16), (8, 20)])
@pytest.mark.parametrize("count", [1, 2, 777, 70001, (1 << 21) + 2])
def test_beaver_mul_trunc_is_mul_then_trunc(n, f, count):
    if n * count * 8 >= 64 << 20 and n not in (5, 8):
        pytest.skip("the streaming variant is covered at n = 5 and 8")
    rng = np.random.default_rng(n * 7 + count)
    xs = rng.integers(-(1 << 28), 1 << 28, size=count, dtype=np.int64).view(np.uint64)
    ys = rng.integers(-(1 << 28), 1 << 28, size=count, dtype=np.int64).view(np.uint64)
    X, Y = oracle.share(xs, n, 31, oracle.STREAM_X), oracle.share(ys, n, 31, oracle.STREAM_Y)
    a, b, c = oracle.dealer_mul(n, count, seed=32)
    r, rt, rm = oracle.trunc_dealer(n, count, f, seed=33)
    want = oracle.trunc(oracle.beaver_mul(X, Y, a, b, c), r, rt, rm, f)
    Xd = dev(X)
    args = (dev(Y), dev(a), dev(b), dev(c), dev(r), dev(rt), dev(rm), f)
    got = spin.beaver_mul_trunc(Xd, *args)
    assert (host(got) == want).all()
    # the opened result is the product shifted down, up to the truncation's one unit (first 1000 elements)
    opened = host(spin.open(got)).view(np.int64)[:1000]
    floors = [(int(p) * int(q)) >> f for p, q in zip(xs.view(np.int64)[:1000], ys.view(np.int64)[:1000])]
    assert set(int(o) - w for o, w in zip(opened, floors)) <= {0, 1}
    spin.beaver_mul_trunc(Xd, *args, out=Xd)                     # in place on the first operand
    assert (host(Xd) == want).all()


# Past 64 MB per call the many-stream kernels switch to non-temporal loads and stores; both the paired
# (even count) and the single-word (odd count) forms of that variant are compared here.
@pytest.mark.parametrize("n,count", [(5, (1 << 21) + 2), (3, (3 << 20) + 1), (8, 1 << 20)])
def test_streaming_variants_of_open_mul_trunc(n, count):
    assert n * count * 8 >= 64 << 20
    rng = np.random.default_rng(n + count)
    f = 16
    xs = rng.integers(-(1 << 40), 1 << 40, size=count, dtype=np.int64).view(np.uint64)
    ys = rng.integers(-(1 << 20), 1 << 20, size=count, dtype=np.int64).view(np.uint64)
    X, Y = oracle.share(xs, n, 11, oracle.STREAM_X), oracle.share(ys, n, 11, oracle.STREAM_Y)
    a, b, c = oracle.dealer_mul(n, count, seed=12)
    r, rt, rm = oracle.trunc_dealer(n, count, f, seed=13)
    Xd = spin.share(dev(xs), n, 11, oracle.STREAM_X)
    assert (host(Xd) == X).all()
    assert (host(spin.open(Xd, dev(a))) == oracle.open_(X, a)).all()
    zo = oracle.beaver_mul(X, Y, a, b, c)
    zd = spin.beaver_mul(Xd, dev(Y), dev(a), dev(b), dev(c))
    assert (host(zd) == zo).all()
    to = oracle.trunc(zo, r, rt, rm, f)
    spin.trunc(zd, dev(r), dev(rt), dev(rm), f, out=zd)
    assert (host(zd) == to).all()
    want = oracle.trunc(oracle.lincomb([X, zo], [3, -5], 77), r, rt, rm, f)
    got = spin.lincomb_trunc([Xd, dev(zo)], [3, -5], 77, f, (dev(r), dev(rt), dev(rm)))
    assert (host(got) == want).all()


# ----------------------------------------------------------------------------- Beaver matmul
def matmul_case(n, batch, M, N, K, seed, path, X=None, Y=None, consistent=True):
    rng = np.random.default_rng(seed)
    if X is None:
        X, Y = rand_u64(rng, (n, batch, M, K)), rand_u64(rng, (n, batch, K, N))
    if consistent:
        A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=seed)
    else:
        A, B, C = rand_u64(rng, X.shape), rand_u64(rng, Y.shape), rand_u64(rng, (n, batch, M, N))
    want = oracle.beaver_matmul(X, Y, A, B, C)
    got = spin.beaver_matmul(dev(X), dev(Y), dev(A), dev(B), dev(C), path=path)
    torch.cuda.synchronize()
    return host(got), want


PATHS = [pytest.param(spin.LIMB_MFMA, id="limb"), pytest.param(spin.VALU, id="valu")]
SHAPES = [(1, 1, 1, 1, 1), (2, 1, 1, 1, 1), (3, 1, 64, 64, 64), (2, 1, 33, 31, 32), (3, 2, 130, 70, 45),
          (1, 1, 128, 64, 32), (5, 1, 129, 65, 33), (8, 1, 40, 40, 40), (4, 3, 17, 200, 100),
          (2, 1, 300, 260, 257), (3, 5, 128, 128, 64), (2, 1, 7, 5, 1000)]


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("n,batch,M,N,K", SHAPES)
def test_beaver_matmul_small_shapes(n, batch, M, N, K, path):
    got, want = matmul_case(n, batch, M, N, K, seed=n * 7 + M, path=path)
    assert (got == want).all()


@pytest.mark.parametrize("path", PATHS)
def test_beaver_matmul_in_place_on_c(path):
    rng = np.random.default_rng(3)
    n, batch, M, N, K = 3, 2, 96, 80, 72
    X, Y = rand_u64(rng, (n, batch, M, K)), rand_u64(rng, (n, batch, K, N))
    A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=3)
    Cd = dev(C)
    spin.beaver_matmul(dev(X), dev(Y), dev(A), dev(B), Cd, path=path, out=Cd)
    assert (host(Cd) == oracle.beaver_matmul(X, Y, A, B, C)).all()


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("n,batch,M,N,K", [(1, 1, 1, 1, 1), (2, 1, 33, 31, 32), (3, 2, 130, 70, 45), (5, 1, 129, 65, 33),
                                           (3, 64, 128, 128, 64), (2, 1, 300, 260, 257), (4, 3, 17, 200, 101)])
def test_beaver_matmul_with_transposed_right_operand(n, batch, M, N, K, path):
    # Y and B handed over as [n][batch][N][K] (the layout of K in Q.K^T); same result as the plain call
    rng = np.random.default_rng(n * 31 + M)
    X, Y = rand_u64(rng, (n, batch, M, K)), rand_u64(rng, (n, batch, K, N))
    A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=n * 31 + M)
    want = oracle.beaver_matmul(X, Y, A, B, C)
    Yt = np.ascontiguousarray(Y.transpose(0, 1, 3, 2))
    Bt = np.ascontiguousarray(B.transpose(0, 1, 3, 2))
    got = spin.beaver_matmul(dev(X), dev(Yt), dev(A), dev(Bt), dev(C), path=path, y_transposed=True)
    assert (host(got) == want).all()


@pytest.mark.parametrize("path", PATHS)
def test_tall_operand_with_more_tile_rows_than_a_grid_axis_holds(path):
    # 65537 tile rows of 64 (VALU path) exceed the 65535 blocks of a grid's y and z axes
    M = 65536 * 64 + 1
    got, want = matmul_case(2, 1, M, 3, 2, seed=21, path=path)
    assert (got == want).all()


@pytest.mark.parametrize("n,batch,M,N,K", [(2, 1, 128, 64, 4096), (3, 1, 200, 130, 1000), (1, 2, 64, 64, 999),
                                           (5, 1, 256, 192, 352), (2, 1, 100, 60, 16352 + 320)])
def test_few_tiles_and_a_long_inner_dimension(n, batch, M, N, K):
    # fewer output tiles than the chip has CUs: several workgroups share a tile, each taking a run of k-steps
    # (runs that start in the first operand pair, straddle the switch, or lie in the second) and adding its
    # part onto Z atomically; out of place (Z first becomes C) and in place on C
    rng = np.random.default_rng(M + K)
    X, Y = rand_u64(rng, (n, batch, M, K)), rand_u64(rng, (n, batch, K, N))
    A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=M + K)
    want = oracle.beaver_matmul(X, Y, A, B, C)
    Xd, Yd, Ad, Bd, Cd = (dev(t) for t in (X, Y, A, B, C))
    got = spin.beaver_matmul(Xd, Yd, Ad, Bd, Cd, path=spin.LIMB_MFMA)
    assert (host(got) == want).all()
    assert (host(Cd) == C).all()                                  # C untouched
    spin.beaver_matmul(Xd, Yd, Ad, Bd, Cd, path=spin.LIMB_MFMA, out=Cd)
    assert (host(Cd) == want).all()
    # repeated calls give the same words (the atomic accumulation is exact, so order cannot matter)
    again = spin.beaver_matmul(Xd, Yd, Ad, Bd, dev(C), path=spin.LIMB_MFMA)
    assert torch.equal(again, got)


# Products with a single column tile (N <= 64) -- or a few and a short inner dimension --, at most three parties
# and an even inner dimension take the row-streaming kernel, which builds the left fragments inside the GEMM: one k-tile, two, three (the LDS ring
# length) and many; ragged rows, columns and inner dimension; batches; in place; transposed right operand.
ROW_SHAPES = [(3, 1, 32, 64, 32), (3, 1, 64, 64, 64), (2, 1, 33, 31, 34), (1, 1, 100, 64, 96), (3, 2, 130, 57, 46),
              (3, 1, 1, 1, 2), (2, 3, 95, 64, 128), (3, 1, 4096, 64, 576), (3, 64, 128, 64, 128), (1, 2, 257, 33, 1000),
              (3, 1, 8192, 64, 70), (2, 1, 9000, 48, 2048), (3, 1, 70, 64, 160), (2, 2, 40, 50, 192), (3, 1, 33, 64, 226),
              # more row blocks than CUs: a workgroup walks several of them, its producer running ahead across the boundary
              (3, 1, 9000, 64, 32), (2, 3, 3000, 130, 40), (1, 1, 20000, 33, 6), (3, 1, 8500, 64, 96), (2, 70, 128, 100, 64),
              # a few column tiles and a short inner dimension (the attention shapes): one pass per column tile
              (3, 64, 128, 128, 64), (3, 2, 100, 130, 40), (2, 1, 64, 192, 32), (3, 8, 196, 196, 64)]


@pytest.mark.parametrize("n,batch,M,N,K", ROW_SHAPES)
def test_beaver_matmul_single_column_tile_shapes(n, batch, M, N, K):
    print("rows case", n, batch, M, N, K, flush=True)
    rng = np.random.default_rng(M * 3 + K)
    X, Y = rand_u64(rng, (n, batch, M, K)), rand_u64(rng, (n, batch, K, N))
    A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=M + N + K)
    want = oracle.beaver_matmul(X, Y, A, B, C)
    Xd, Yd, Ad, Bd, Cd = (dev(t) for t in (X, Y, A, B, C))
    got = spin.beaver_matmul(Xd, Yd, Ad, Bd, Cd, path=spin.LIMB_MFMA)
    assert (host(got) == want).all()
    assert (host(Cd) == C).all()
    Bt = dev(np.ascontiguousarray(B.transpose(0, 1, 3, 2)))
    Yt = dev(np.ascontiguousarray(Y.transpose(0, 1, 3, 2)))
    assert torch.equal(spin.beaver_matmul(Xd, Yt, Ad, Bt, Cd, path=spin.LIMB_MFMA, y_transposed=True), got)
    spin.beaver_matmul(Xd, Yd, Ad, Bd, Cd, path=spin.LIMB_MFMA, out=Cd)          # in place on C
    assert (host(Cd) == want).all()


def test_single_column_tile_worst_case_digits():
    # all digits -128 in every operand of both products, at the longest inner dimension the row kernel accumulates
    # in one launch (511 k-tiles): the int32 partial sums run at their proven extreme
    n, M, N, K = 2, 300, 64, 511 * 32
    worst = np.uint64(0x7F7F7F7F7F7F7F80)
    X = np.zeros((n, 1, M, K), dtype=np.uint64); X[:] = worst
    Y = np.zeros((n, 1, K, N), dtype=np.uint64); Y[:] = worst
    A = np.zeros_like(X); B = np.zeros_like(Y); A[1] = worst; B[1] = worst
    C = np.zeros((n, 1, M, N), dtype=np.uint64)
    want = oracle.beaver_matmul(X, Y, A, B, C)
    got = spin.beaver_matmul(dev(X), dev(Y), dev(A), dev(B), dev(C), path=spin.LIMB_MFMA)
    assert (host(got) == want).all()


def test_limb_path_worst_case_digits_and_inner_dimension_split():
    # every digit of every operand equal to -128 (value 0x7F7F7F7F7F7F7F80), with K large enough that
    # the inner dimension is split into more than one accumulation chunk: the int32 partial sums run
    # at their proven extreme.  E = X - A and F = Y - B are forced to that value with zero triples.
    n, M, N, K = 2, 32, 32, 16352 + 96
    worst = np.uint64(0x7F7F7F7F7F7F7F80)
    X = np.zeros((n, 1, M, K), dtype=np.uint64); X[0] = worst
    Y = np.zeros((n, 1, K, N), dtype=np.uint64); Y[0] = worst
    A = np.zeros_like(X); B = np.zeros_like(Y); A[1] = worst; B[1] = worst   # A_1.F and E.B_1 extreme too
    X[1] = worst; Y[1] = worst                                               # so that E = F = worst
    C = np.zeros((n, 1, M, N), dtype=np.uint64)
    want = oracle.beaver_matmul(X, Y, A, B, C)
    got = spin.beaver_matmul(dev(X), dev(Y), dev(A), dev(B), dev(C), path=spin.LIMB_MFMA)
    assert (host(got) == want).all()
    # and random data across the split
    got, want = matmul_case(2, 1, 40, 36, 16352 + 40, seed=9, path=spin.LIMB_MFMA, consistent=False)
    assert (got == want).all()


def encode_share(x, n, f, seed, stream):
    return oracle.share(oracle.encode(x, f), n, seed, stream)


def fixed_point_pipeline(cfg, gemm_index, X_real, Y_real, path, rows=None, cross_path=None):
    """share -> Beaver matmul -> trunc on the GPU vs the oracle; returns the largest decoded error.
    rows = None compares whole tensors.  cross_path: a second GEMM path whose whole Z must equal the first's."""
    c = workloads.CONFIGS[cfg]
    n, f = c.n, c.f
    batch, M, K = X_real.shape
    N = Y_real.shape[2]
    xe, ye = oracle.encode(X_real, f), oracle.encode(Y_real, f)
    # sharing on the GPU must equal the oracle's sharing
    Xd = spin.share(dev(xe), n, c.seed, oracle.STREAM_X)
    Yd = spin.share(dev(ye), n, c.seed, oracle.STREAM_Y)
    X, Y = oracle.share(xe, n, c.seed, oracle.STREAM_X), oracle.share(ye, n, c.seed, oracle.STREAM_Y)
    assert (host(Xd) == X).all() and (host(Yd) == Y).all()
    A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=c.seed)
    Ad, Bd, Cd = dev(A), dev(B), dev(C)
    Zd = spin.beaver_matmul(Xd, Yd, Ad, Bd, Cd, path=path)
    if cross_path is not None:
        assert torch.equal(Zd, spin.beaver_matmul(Xd, Yd, Ad, Bd, Cd, path=cross_path))
    del Ad, Bd, Cd
    Zg = host(Zd)
    if rows is None:
        Zo = oracle.beaver_matmul(X, Y, A, B, C)
        assert (Zg == Zo).all()
        sel = slice(None)
    else:
        Zo = oracle.beaver_matmul(X, Y, A, B, C, rows=rows)
        assert (Zg[:, :, rows] == Zo).all()
        sel = rows
    # reconstruction: the shares sum to the plain ring product (plain definition, on the checked rows)
    zsum = Zg.sum(axis=0, dtype=np.uint64)
    for b in range(batch):
        assert (zsum[b][sel] == oracle.ring_matmul(xe[b][sel], ye[b])).all()
    r, rt, rm = oracle.trunc_dealer(n, batch * M * N, f, seed=c.seed)
    Td = spin.trunc(Zd.view(n, -1), dev(r), dev(rt), dev(rm), f)
    Tg = host(Td).reshape(n, batch, M, N)
    if rows is None:
        assert (Tg == oracle.trunc(Zo.reshape(n, -1), r, rt, rm, f).reshape(Tg.shape)).all()
    else:
        idx = (np.arange(batch)[:, None, None] * M + np.asarray(rows)[None, :, None]) * N + np.arange(N)
        idx = idx.reshape(-1)
        want = oracle.trunc(Zo.reshape(n, -1), r[:, idx], rt[:, idx], rm[:, idx], f)
        assert (Tg[:, :, rows].reshape(n, -1) == want).all()
    got = oracle.decode(host(spin.open(Td)).reshape(batch, M, N), f)
    ref = np.matmul(X_real, Y_real)
    err = np.abs(got - ref)[:, sel].max()
    assert err <= 2.0 ** -f * (K + 2), err
    return err


@pytest.mark.parametrize("path", PATHS)
def test_config1_full(path):
    X, Y = workloads.gemm_plaintexts(1)
    fixed_point_pipeline(1, 0, X, Y, path)


@pytest.mark.parametrize("path", PATHS)
def test_config2_gemm_full(path):
    X, Y = workloads.gemm_plaintexts(2)
    fixed_point_pipeline(2, 0, X, Y, path)


def test_config2_vectors_full():
    c = workloads.CONFIGS[2]
    n, f, L = c.n, c.f, c.vec
    xr, yr = workloads.vec_plaintexts(2)
    X, Y = encode_share(xr, n, f, c.seed, oracle.STREAM_X), encode_share(yr, n, f, c.seed, oracle.STREAM_Y)
    a, b, cc = oracle.dealer_mul(n, L, seed=c.seed)
    r, rt, rm = oracle.trunc_dealer(n, L, f, seed=c.seed)
    zd = spin.beaver_mul(dev(X), dev(Y), dev(a), dev(b), dev(cc))
    zo = oracle.beaver_mul(X, Y, a, b, cc)
    assert (host(zd) == zo).all()
    td = spin.trunc(zd, dev(r), dev(rt), dev(rm), f)
    assert (host(td) == oracle.trunc(zo, r, rt, rm, f)).all()
    got = oracle.decode(host(spin.open(td)), f)
    assert np.abs(got - xr * yr).max() <= 2.0 ** -f * (1 + 2) * max(1.0, np.abs(xr).max(), np.abs(yr).max())


@pytest.mark.parametrize("path", PATHS)
def test_config3_conv_shape_eighth_batch(path):
    # 16 of the 128 images: M = 16384 rows of the same K = 576, N = 64 GEMM, every row checked
    X, Y = workloads.gemm_plaintexts(3, scale=16 / 128)
    assert X.shape == (1, 16384, 576)
    fixed_point_pipeline(3, 0, X, Y, path)


def test_config3_conv_shape_full():
    # the whole 131072 x 576 x 64 product of 3 parties, the launch the benchmark times: every share word of Z and
    # of the truncated Z against the oracle, the reconstruction and the decoded bound over every row
    X, Y = workloads.gemm_plaintexts(3)
    assert X.shape == (1, 131072, 576)
    fixed_point_pipeline(3, 0, X, Y, spin.LIMB_MFMA, cross_path=spin.VALU)


@pytest.mark.parametrize("path", PATHS)
def test_config4_attention_full(path):
    c = workloads.CONFIGS[4]
    n, f = c.n, c.f
    Q, KT = workloads.gemm_plaintexts(4, 0)                 # [64,128,64], [64,64,128]  (K already transposed)
    fixed_point_pipeline(4, 0, Q, KT, path)
    # P.V with P = decoded truncated scores scaled into a softmax-like range (no softmax: Section 7 is out of scope)
    P = np.matmul(Q, KT) / 64.0
    _, V = workloads.gemm_plaintexts(4, 1)
    fixed_point_pipeline(4, 1, P, V, path)


def test_config4_score_tensor_elementwise():
    c = workloads.CONFIGS[4]
    n, f, L = c.n, c.f, c.vec
    xr, yr = workloads.vec_plaintexts(4)
    X, Y = encode_share(xr, n, f, c.seed, oracle.STREAM_X), encode_share(yr, n, f, c.seed, oracle.STREAM_Y)
    a, b, cc = oracle.dealer_mul(n, L, seed=c.seed)
    zo = oracle.beaver_mul(X, Y, a, b, cc)
    assert (host(spin.beaver_mul(dev(X), dev(Y), dev(a), dev(b), dev(cc))) == zo).all()


def test_config5_full():
    # 5 parties, 4096^3, the launch the benchmark times, compared whole: every one of the 5 x 2^24 share words of
    # Z and of the truncated Z against the oracle (about 8e11 ring multiply-adds on the host cores), the sum of
    # the shares against the plain ring product, the decoded result against float64 over every row, and the
    # baseline GEMM path against the limb path over the whole of Z.
    X, Y = workloads.gemm_plaintexts(5)
    fixed_point_pipeline(5, 0, X, Y, spin.LIMB_MFMA, cross_path=spin.VALU)


def test_paths_agree_on_config5_shape_slice():
    # both GEMM paths on a 5-party 512 x 4096 x 4096 slice, full comparison against each other
    rng = np.random.default_rng(56)
    n, M, N, K = 5, 512, 512, 4096
    X, Y = dev(rand_u64(rng, (n, 1, M, K))), dev(rand_u64(rng, (n, 1, K, N)))
    A, B, C = dev(rand_u64(rng, (n, 1, M, K))), dev(rand_u64(rng, (n, 1, K, N))), dev(rand_u64(rng, (n, 1, M, N)))
    z0 = spin.beaver_matmul(X, Y, A, B, C, path=spin.LIMB_MFMA)
    z1 = spin.beaver_matmul(X, Y, A, B, C, path=spin.VALU)
    assert torch.equal(z0, z1)


@pytest.mark.parametrize("n", [4, 6, 7, 8])
def test_every_party_count_at_a_multi_tile_size(n):
    # 512 x 384 x 640: several workgroup tiles and 20 k-tiles per operand pair; both paths against each other,
    # sampled rows against the oracle, and the truncated result through the fused open
    M, N, K, f = 512, 384, 640, 16
    rng = np.random.default_rng(80 + n)
    X, Y = rand_u64(rng, (n, 1, M, K)), rand_u64(rng, (n, 1, K, N))
    A, B, C = oracle.dealer_matmul(n, 1, M, N, K, seed=80 + n)
    args = [dev(t) for t in (X, Y, A, B, C)]
    zl = spin.beaver_matmul(*args, path=spin.LIMB_MFMA)
    zv = spin.beaver_matmul(*args, path=spin.VALU)
    assert torch.equal(zl, zv)
    rows = np.sort(rng.choice(M, 48, replace=False)); rows[0], rows[-1] = 0, M - 1
    assert (host(zl)[:, :, rows] == oracle.beaver_matmul(X, Y, A, B, C, rows=rows)).all()
    r, rt, rm = oracle.trunc_dealer(n, M * N, f, seed=81 + n)
    got = host(spin.trunc(zl.view(n, -1), dev(r), dev(rt), dev(rm), f)).reshape(n, M, N)[:, rows]
    idx = (np.asarray(rows)[:, None] * N + np.arange(N)).reshape(-1)
    want = oracle.trunc(host(zl).reshape(n, -1)[:, idx], r[:, idx], rt[:, idx], rm[:, idx], f)
    assert (got.reshape(n, -1) == want).all()


def test_calls_run_on_the_callers_stream():
    # the whole path enqueued on a side stream, with no synchronisation until the end: every call must be
    # ordered on that stream (a kernel launched on another stream would read unfinished inputs)
    rng = np.random.default_rng(77)
    n, M, N, K, f = 3, 257, 130, 96, 16
    x = rng.integers(-(1 << 20), 1 << 20, size=(1, M, K), dtype=np.int64).view(np.uint64)
    y = rng.integers(-(1 << 20), 1 << 20, size=(1, K, N), dtype=np.int64).view(np.uint64)
    A, B, C = oracle.dealer_matmul(n, 1, M, N, K, seed=78)
    r, rt, rm = oracle.trunc_dealer(n, M * N, f, seed=78)
    xd, yd, Ad, Bd, Cd, rd, rtd, rmd = map(dev, (x, y, A, B, C, r, rt, rm))
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for path in (spin.LIMB_MFMA, spin.VALU):
            Xs = spin.share(xd, n, 78, oracle.STREAM_X)
            Ys = spin.share(yd, n, 78, oracle.STREAM_Y)
            Z = spin.beaver_matmul(Xs, Ys, Ad, Bd, Cd, path=path)
            T = spin.trunc(Z.view(n, -1), rd, rtd, rmd, f)
            out = spin.open(T)
    side.synchronize()
    X, Y = oracle.share(x, n, 78, oracle.STREAM_X), oracle.share(y, n, 78, oracle.STREAM_Y)
    Zo = oracle.beaver_matmul(X, Y, A, B, C)
    To = oracle.trunc(Zo.reshape(n, -1), r, rt, rm, f)
    assert (host(T) == To).all() and (host(out) == oracle.open_(To)).all()
