"""Randomised pins of the oracle against Python integers, over ring widths, party counts and shapes that the
fixed cases do not enumerate (hypothesis draws them; the seed database is not used, every run is fresh but
bounded).  Each property restates the protocol step in exact integer arithmetic, independently of the C code."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle

RING = st.sampled_from([8, 13, 16, 32, 47, 64])


def ints(a):
    return [int(v) for v in np.asarray(a).reshape(-1)]


@settings(max_examples=60, deadline=None)
@given(l=RING, n=st.integers(1, 5), M=st.integers(1, 4), N=st.integers(1, 4), K=st.integers(1, 5),
       seed=st.integers(0, 2 ** 32))
def test_beaver_matmul_shares_in_integers(l, n, M, N, K, seed):
    mod = 1 << l
    rng = np.random.default_rng(seed)
    X = rng.integers(0, mod, size=(n, 1, M, K), dtype=np.uint64) if l < 64 else rng.integers(0, 1 << 64, size=(n, 1, M, K), dtype=np.uint64)
    Y = rng.integers(0, mod, size=(n, 1, K, N), dtype=np.uint64) if l < 64 else rng.integers(0, 1 << 64, size=(n, 1, K, N), dtype=np.uint64)
    A, B, C = oracle.dealer_matmul(n, 1, M, N, K, seed=seed, l=l)
    Z = oracle.beaver_matmul(X, Y, A, B, C, l=l)
    x = [[sum(int(X[i, 0, m, k]) for i in range(n)) % mod for k in range(K)] for m in range(M)]
    y = [[sum(int(Y[i, 0, k, q]) for i in range(n)) % mod for q in range(N)] for k in range(K)]
    a = [[sum(int(A[i, 0, m, k]) for i in range(n)) % mod for k in range(K)] for m in range(M)]
    b = [[sum(int(B[i, 0, k, q]) for i in range(n)) % mod for q in range(N)] for k in range(K)]
    for m in range(M):
        for q in range(N):
            # the triple and the reconstruction
            assert sum(int(C[i, 0, m, q]) for i in range(n)) % mod == sum(a[m][k] * b[k][q] for k in range(K)) % mod
            assert sum(int(Z[i, 0, m, q]) for i in range(n)) % mod == sum(x[m][k] * y[k][q] for k in range(K)) % mod
            for i in range(n):
                v = int(C[i, 0, m, q])
                for k in range(K):
                    e, f = (x[m][k] - a[m][k]) % mod, (y[k][q] - b[k][q]) % mod
                    v += e * int(B[i, 0, k, q]) + int(A[i, 0, m, k]) * f + (e * f if i == 0 else 0)
                assert v % mod == int(Z[i, 0, m, q])


@settings(max_examples=80, deadline=None)
@given(l=RING, n=st.integers(1, 5), data=st.data())
def test_truncation_closed_form_in_integers(l, n, data):
    f = data.draw(st.integers(1, l - 3))
    seed = data.draw(st.integers(0, 2 ** 32))
    count = 40
    mod, half = 1 << l, 1 << (l - 2)
    rng = np.random.default_rng(seed)
    xs = [int(v) for v in rng.integers(-half, half, size=count)] if l < 64 else \
        [int(v) for v in rng.integers(-(1 << 62), 1 << 62, size=count)]
    xs[0], xs[1] = -half, half - 1
    X = oracle.share(np.array([v % mod for v in xs], dtype=np.uint64), n, seed, oracle.STREAM_X, l=l)
    r, rt, rm = oracle.trunc_dealer(n, count, f, seed=seed + 1, l=l)
    out = ints(oracle.open_(oracle.trunc(X, r, rt, rm, f, l=l), l=l))
    rr = ints(oracle.open_(r, l=l))
    for k in range(count):
        xp = xs[k] + half
        v = ((xp % (1 << f)) + (rr[k] % (1 << f))) >> f
        assert out[k] == ((xs[k] >> f) + v) % mod


@settings(max_examples=60, deadline=None)
@given(l=RING, n=st.integers(1, 6), count=st.integers(1, 30), seed=st.integers(0, 2 ** 32))
def test_elementwise_update_in_integers(l, n, count, seed):
    mod = 1 << l
    rng = np.random.default_rng(seed)
    hi = mod if l < 64 else 1 << 64
    X = rng.integers(0, hi, size=(n, count), dtype=np.uint64)
    Y = rng.integers(0, hi, size=(n, count), dtype=np.uint64)
    a, b, c = oracle.dealer_mul(n, count, seed=seed, l=l)
    z = oracle.beaver_mul(X, Y, a, b, c, l=l)
    for k in range(count):
        e = sum(int(X[i, k]) - int(a[i, k]) for i in range(n)) % mod
        f = sum(int(Y[i, k]) - int(b[i, k]) for i in range(n)) % mod
        assert sum(int(c[i, k]) for i in range(n)) % mod == \
            (sum(int(a[i, k]) for i in range(n)) * sum(int(b[i, k]) for i in range(n))) % mod
        for i in range(n):
            want = int(c[i, k]) + e * int(b[i, k]) + int(a[i, k]) * f + (e * f if i == 0 else 0)
            assert want % mod == int(z[i, k])
