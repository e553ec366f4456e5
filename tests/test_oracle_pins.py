"""Pins of the CPU oracle against things other than itself: published vectors,
the paper's worked encoding example, closed forms, Python big-integer
arithmetic, numpy's wrapping uint64 matmul, and exhaustive brute force over
tiny rings.  Every function of oracle/spin_oracle.c is held by at least one."""
import os

import numpy as np
import pytest

import oracle

M64 = (1 << 64) - 1
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def big(a):
    """numpy uint64 array -> nested Python ints."""
    return np.asarray(a, dtype=np.uint64).astype(object)


def signed(v, l):
    v &= (1 << l) - 1
    return v - (1 << l) if v >> (l - 1) else v


# --------------------------------------------------------------------------- generator
def test_generator_step_matches_published_splitmix64_sequences():
    # SplitMix64 reference outputs (Steele, Lea, Flood 2014; Vigna's splitmix64.c test values):
    # state 1234567 and state 0.
    want = [6457827717110365317, 3203168211198807973, 9817491932198370423,
            4593380528125082431, 16408922859458223821]
    assert [oracle.absorb(1234567, i) for i in range(5)] == want
    assert [oracle.absorb(0, i) for i in range(3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4,
                                                       0x06C45D188009454F]


def test_rand64_matches_big_integer_evaluation_of_the_spec():
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "rng_vectors.txt")) if not ln.startswith("#")]
    assert len(rows) >= 10
    for seed, stream, party, idx, val in rows:
        assert oracle.rand64(int(seed, 16), int(stream, 16), int(party, 16), int(idx, 16)) == int(val, 16)


def test_rand64_streams_are_distinct_and_balanced():
    vals = np.array([oracle.rand64(9, s, p, k) for s in range(1, 4) for p in range(3) for k in range(400)],
                    dtype=np.uint64)
    assert len(set(vals.tolist())) == vals.size
    bits = np.unpackbits(vals.view(np.uint8)).mean()
    assert abs(bits - 0.5) < 0.01


# --------------------------------------------------------------------------- encoding (Section 4.1)
def test_encode_paper_example_and_floor():
    # [7.7]_p = floor(7.7 * 2^p): the paper's example, at p = 16 -> 504627 (7.7*65536 = 504627.2)
    assert oracle.encode([7.7], 16)[0] == 504627
    # floor goes toward minus infinity and lands in two's complement
    assert oracle.encode([-7.7], 16)[0] == (1 << 64) - 504628
    assert oracle.encode([-1e-9], 16)[0] == M64
    assert oracle.encode([0.0, 1.0, -1.0], 16).tolist() == [0, 65536, (1 << 64) - 65536]


def test_encode_decode_round_trip_interval():
    rng = np.random.default_rng(1)
    x = rng.normal(0, 100, size=5000)
    for p in (8, 16, 26):
        back = oracle.decode(oracle.encode(x, p), p)
        assert np.all(back <= x) and np.all(back > x - 2.0 ** -p)


def test_decode_reads_small_rings_as_signed():
    assert oracle.decode(np.array([0xFF, 0x80, 0x7F], dtype=np.uint64), 0, l=8).tolist() == [-1.0, -128.0, 127.0]


# --------------------------------------------------------------------------- share / open (Section 4.1)
@pytest.mark.parametrize("n", [1, 2, 3, 5, 8])
def test_share_reconstructs_and_uses_the_generator(n):
    rng = np.random.default_rng(n)
    x = rng.integers(0, 1 << 64, size=257, dtype=np.uint64)
    sh = oracle.share(x, n, seed=77, stream=oracle.STREAM_X)
    total = sum(big(sh[i]) for i in range(n)) % (1 << 64)
    assert (total == big(x)).all()
    for i in range(1, n):
        assert sh[i, 5] == oracle.rand64(77, oracle.STREAM_X, i, 5)
    if n == 1:
        assert (sh[0] == x).all()
    assert (oracle.open_(sh) == x).all()


def test_open_with_mask_is_sum_of_differences():
    rng = np.random.default_rng(3)
    s = rng.integers(0, 1 << 64, size=(3, 100), dtype=np.uint64)
    m = rng.integers(0, 1 << 64, size=(3, 100), dtype=np.uint64)
    want = (sum(big(s[i]) - big(m[i]) for i in range(3))) % (1 << 64)
    assert (big(oracle.open_(s, m)) == want).all()


# --------------------------------------------------------------------------- ring matmul
def bigint_matmul(P, Q, l=64):
    P, Q = big(P), big(Q)
    M, K = P.shape
    N = Q.shape[1]
    return np.array([[sum(int(P[m, k]) * int(Q[k, q]) for k in range(K)) % (1 << l) for q in range(N)]
                     for m in range(M)], dtype=object)


def test_ring_matmul_against_big_integers_and_numpy():
    rng = np.random.default_rng(5)
    P = rng.integers(0, 1 << 64, size=(7, 9), dtype=np.uint64)
    Q = rng.integers(0, 1 << 64, size=(9, 5), dtype=np.uint64)
    got = oracle.ring_matmul(P, Q)
    assert (big(got) == bigint_matmul(P, Q)).all()
    # non-square operands: a transposed operand or swapped factors cannot give this
    P = rng.integers(0, 1 << 64, size=(65, 130), dtype=np.uint64)
    Q = rng.integers(0, 1 << 64, size=(130, 33), dtype=np.uint64)
    assert (oracle.ring_matmul(P, Q) == P @ Q).all()       # numpy uint64 matmul wraps mod 2^64
    # identity and a permutation: closed forms
    I = np.eye(9, dtype=np.uint64)
    assert (oracle.ring_matmul(I, Q[:9]) == Q[:9]).all()


# --------------------------------------------------------------------------- dealer (Section 4.2)
def test_matmul_triple_is_consistent():
    n, batch, M, N, K = 3, 2, 6, 5, 7
    A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=11)
    a, b, c = (sum(big(T[i]) for i in range(n)) % (1 << 64) for T in (A, B, C))
    for bb in range(batch):
        assert (c[bb] == bigint_matmul(a[bb], b[bb])).all()
    # operand shares are raw generator output
    assert A[2, 1, 3, 4] == oracle.rand64(11, oracle.STREAM_A, 2, (1 * M + 3) * K + 4)
    assert B[1, 0, 2, 1] == oracle.rand64(11, oracle.STREAM_B, 1, 2 * N + 1)


def test_matmul_triple_medium_against_numpy():
    n, batch, M, N, K = 2, 1, 96, 80, 130
    A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=12)
    a, b, c = A.sum(axis=0, dtype=np.uint64), B.sum(axis=0, dtype=np.uint64), C.sum(axis=0, dtype=np.uint64)
    assert (c[0] == a[0] @ b[0]).all()


def test_elementwise_triple_is_consistent():
    a, b, c = oracle.dealer_mul(5, 1000, seed=13)
    av, bv, cv = (sum(big(t[i]) for i in range(5)) % (1 << 64) for t in (a, b, c))
    assert (cv == (av * bv) % (1 << 64)).all()


# --------------------------------------------------------------------------- Beaver multiplication (Section 4.3)
@pytest.mark.parametrize("n", [1, 2, 3, 5])
def test_beaver_matmul_reconstructs_plain_product(n):
    rng = np.random.default_rng(20 + n)
    batch, M, N, K = 2, 9, 6, 11
    x = rng.integers(0, 1 << 64, size=(batch, M, K), dtype=np.uint64)
    y = rng.integers(0, 1 << 64, size=(batch, K, N), dtype=np.uint64)
    X = oracle.share(x, n, 31, oracle.STREAM_X)
    Y = oracle.share(y, n, 31, oracle.STREAM_Y)
    A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=31)
    Z, E, F = oracle.beaver_matmul(X, Y, A, B, C, return_opened=True)
    z = sum(big(Z[i]) for i in range(n)) % (1 << 64)
    for bb in range(batch):
        assert (z[bb] == bigint_matmul(x[bb], y[bb])).all()
    # the opened values are X-A and Y-B
    a = sum(big(A[i]) for i in range(n))
    assert (big(E) == (big(x) - a) % (1 << 64)).all()
    # every share follows its own formula (big integers), not just the sum
    for i in range(n):
        for bb in range(batch):
            want = (big(C[i, bb]) + bigint_matmul(E[bb], B[i, bb]) + bigint_matmul(A[i, bb], F[bb])
                    + (bigint_matmul(E[bb], F[bb]) if i == 0 else 0)) % (1 << 64)
            assert (big(Z[i, bb]) == want).all()


def test_beaver_matmul_single_party_is_textbook_matmul():
    rng = np.random.default_rng(40)
    x = rng.integers(0, 1 << 64, size=(1, 1, 33, 17), dtype=np.uint64)
    y = rng.integers(0, 1 << 64, size=(1, 1, 17, 29), dtype=np.uint64)
    A, B, C = oracle.dealer_matmul(1, 1, 33, 29, 17, seed=41)
    Z = oracle.beaver_matmul(x, y, A, B, C)
    assert (Z[0, 0] == x[0, 0] @ y[0, 0]).all()


def test_beaver_matmul_row_subset_equals_full_rows():
    rng = np.random.default_rng(42)
    n, batch, M, N, K = 3, 2, 20, 7, 13
    X = rng.integers(0, 1 << 64, size=(n, batch, M, K), dtype=np.uint64)
    Y = rng.integers(0, 1 << 64, size=(n, batch, K, N), dtype=np.uint64)
    A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=43)
    rows = np.array([19, 0, 7])
    assert (oracle.beaver_matmul(X, Y, A, B, C, rows=rows) == oracle.beaver_matmul(X, Y, A, B, C)[:, :, rows]).all()


def test_beaver_matmul_share_randomness_does_not_move_the_sum():
    rng = np.random.default_rng(44)
    n, M, N, K = 3, 5, 4, 6
    X = rng.integers(0, 1 << 64, size=(n, 1, M, K), dtype=np.uint64)
    Y = rng.integers(0, 1 << 64, size=(n, 1, K, N), dtype=np.uint64)
    A, B, C = oracle.dealer_matmul(n, 1, M, N, K, seed=45)
    C2 = oracle.share(oracle.open_(C), n, 999, 123)          # same C, different masks
    Z1, Z2 = oracle.beaver_matmul(X, Y, A, B, C), oracle.beaver_matmul(X, Y, A, B, C2)
    assert not (Z1 == Z2).all()
    assert (oracle.open_(Z1) == oracle.open_(Z2)).all()


@pytest.mark.parametrize("n", [2, 3])
def test_beaver_mul_exhaustive_on_a_4_bit_ring(n):
    # every (x, y, a, b) in Z_16^4, random sharings: the shares must sum to x*y mod 16
    l, q = 4, 16
    g = np.arange(q, dtype=np.uint64)
    x, y, a, b = (v.ravel() for v in np.meshgrid(g, g, g, g, indexing="ij"))
    rng = np.random.default_rng(50 + n)

    def split(v):
        parts = rng.integers(0, q, size=(n - 1, v.size), dtype=np.uint64)
        return np.concatenate([((v - parts.sum(axis=0, dtype=np.uint64)) % q)[None], parts])
    xs, ys, as_, bs, cs = split(x), split(y), split(a), split(b), split((a * b) % q)
    z = oracle.beaver_mul(xs, ys, as_, bs, cs, l=l)
    assert z.max() < q
    assert ((z.sum(axis=0, dtype=np.uint64) % q) == (x * y) % q).all()
    # a 1x1x1 matrix product is the same thing
    sel = rng.choice(x.size, 300, replace=False)
    Zm = oracle.beaver_matmul(xs[:, sel].reshape(n, -1, 1, 1), ys[:, sel].reshape(n, -1, 1, 1),
                              as_[:, sel].reshape(n, -1, 1, 1), bs[:, sel].reshape(n, -1, 1, 1),
                              cs[:, sel].reshape(n, -1, 1, 1), l=l)
    assert (Zm.reshape(n, -1) == z[:, sel]).all()


def test_beaver_mul_64_bit_against_big_integers():
    rng = np.random.default_rng(60)
    n, L = 5, 300
    x = rng.integers(0, 1 << 64, size=L, dtype=np.uint64)
    y = rng.integers(0, 1 << 64, size=L, dtype=np.uint64)
    xs, ys = oracle.share(x, n, 61, 1), oracle.share(y, n, 61, 2)
    a, b, c = oracle.dealer_mul(n, L, seed=61)
    z = oracle.beaver_mul(xs, ys, a, b, c)
    assert ((sum(big(z[i]) for i in range(n)) % (1 << 64)) == (big(x) * big(y)) % (1 << 64)).all()
    e = (big(x) - sum(big(a[i]) for i in range(n))) % (1 << 64)
    f = (big(y) - sum(big(b[i]) for i in range(n))) % (1 << 64)
    for i in range(n):
        want = (big(c[i]) + e * big(b[i]) + big(a[i]) * f + (e * f if i == 0 else 0)) % (1 << 64)
        assert (big(z[i]) == want).all()


# --------------------------------------------------------------------------- truncation (Section 4.4)
@pytest.mark.parametrize("n", [2, 3])
def test_trunc_exhaustive_on_an_8_bit_ring(n):
    # l = 8, f = 3: every admissible x in [-2^(l-2), 2^(l-2)-1] with every mask r in Z_256.
    l, f, q = 8, 3, 256
    xs = np.arange(-64, 64)
    rs = np.arange(q)
    x, r = (v.ravel() for v in np.meshgrid(xs, rs, indexing="ij"))
    rng = np.random.default_rng(70 + n)

    def split(v):
        v = np.asarray(v, dtype=np.int64) % q
        parts = rng.integers(0, q, size=(n - 1, v.size), dtype=np.int64)
        return np.concatenate([((v - parts.sum(axis=0)) % q)[None], parts]).astype(np.uint64)
    r_top = (r >> f) & ((1 << (l - 1 - f)) - 1)
    r_msb = r >> (l - 1)
    out = oracle.trunc(split(x), split(r), split(r_top), split(r_msb), f, l=l)
    got = out.sum(axis=0, dtype=np.uint64).astype(np.int64) % q
    got = np.where(got >= q // 2, got - q, got)
    xprime = x + (1 << (l - 2))
    v = ((xprime % (1 << f)) + (r % (1 << f))) >= (1 << f)
    want = (x >> f) + v                                  # arithmetic shift = floor
    assert (got == want).all()
    assert np.abs(got - x / 2.0 ** f).max() < 1.0 + 1e-12   # within one unit of the exact quotient


def test_trunc_dealer_tuple_is_consistent():
    n, L, f = 3, 500, 16
    r, rt, rm = oracle.trunc_dealer(n, L, f, seed=80)
    rv, tv, mv = (sum(big(t[i]) for i in range(n)) % (1 << 64) for t in (r, rt, rm))
    assert (tv == (rv >> f) % (1 << (63 - f))).all()
    assert (mv == rv >> 63).all()
    assert r[1, 7] == oracle.rand64(80, oracle.STREAM_R, 1, 7)
    assert r[0, 7] == oracle.rand64(80, oracle.STREAM_R, 0, 7)
    assert rt[2, 7] == oracle.rand64(80, oracle.STREAM_RTOP, 2, 7)
    assert 0.4 < float(np.mean([int(v) for v in mv])) < 0.6


@pytest.mark.parametrize("n,f", [(2, 16), (3, 16), (5, 26), (3, 1), (2, 61)])
def test_trunc_64_bit_closed_form(n, f):
    rng = np.random.default_rng(90 + n + f)
    L = 4000
    xs = rng.integers(-(1 << 62), 1 << 62, size=L, dtype=np.int64)
    xs[:4] = [-(1 << 62), (1 << 62) - 1, 0, -1]           # the ends of the admissible range
    X = oracle.share(xs.view(np.uint64), n, 91, oracle.STREAM_X)
    r, rt, rm = oracle.trunc_dealer(n, L, f, seed=91)
    out = oracle.trunc(X, r, rt, rm, f)
    got = sum(big(out[i]) for i in range(n)) % (1 << 64)
    rv = sum(big(r[i]) for i in range(n)) % (1 << 64)
    vs = []
    for k in range(L):
        x = int(xs[k])
        v = ((x + (1 << 62)) % (1 << f)) + (int(rv[k]) % (1 << f)) >= (1 << f)
        assert signed(int(got[k]), 64) == (x >> f) + v
        vs.append(v)
    if f == 16:
        # P(v=1) = (x' mod 2^f) / 2^f on average 1/2 for these x
        assert 0.45 < np.mean(vs) < 0.55


@pytest.mark.parametrize("n,f,l", [(2, 16, 64), (3, 16, 64), (5, 26, 64), (3, 1, 64), (2, 61, 64), (3, 3, 8), (4, 5, 16)])
def test_trunc_every_partys_share_against_python_integers(n, f, l):
    # The sum alone does not fix which party adds the public terms.  Section 4.4's signed wrapper around the
    # mask-and-open UnsignedTruncate, with the reading that party 0 (the paper's party 1) adds every public
    # term, written out per party in exact integers:
    #   c = sum_i (x_i + r_i) + 2^(l-2);  c_msb = bit l-1 of c;  c' = bits f..l-2 of c
    #   out_i = -r_top_i + 2^(l-1-f) (r_msb_i - 2 c_msb r_msb_i)              for every party, and
    #   out_0 += c' + 2^(l-1-f) c_msb - 2^(l-2-f)                              for party 0 only.
    q = 1 << l
    rng = np.random.default_rng(1000 * n + 10 * f + l)
    L = 300
    X, R, RT, RM = (rng.integers(0, q, size=(n, L), dtype=np.uint64) for _ in range(4))   # arbitrary share words
    out = oracle.trunc(X, R, RT, RM, f, l=l)
    for k in range(L):
        x, r, rt, rm = ([int(t[i, k]) for i in range(n)] for t in (X, R, RT, RM))
        c = (sum(x) + sum(r) + (1 << (l - 2))) % q
        c_msb = c >> (l - 1)
        c_top = (c >> f) % (1 << (l - 1 - f))
        for i in range(n):
            want = -rt[i] + (1 << (l - 1 - f)) * (rm[i] - 2 * c_msb * rm[i])
            if i == 0:
                want += c_top + (1 << (l - 1 - f)) * c_msb - (1 << (l - 2 - f))
            assert int(out[i, k]) == want % q, (i, k)


def test_trunc_out_of_range_input_is_wrong_as_the_paper_warns():
    # x outside [-2^(l-2), 2^(l-2)-1] makes x + 2^(l-2) use the top bit and UnsignedTruncate stops
    # working (Section 4.4).  On l = 8, f = 3, x = 100: x' = 164 = 128 + 36, and the result is off by
    # 2^(l-f) exactly when 36 + (r mod 128) carries into the top bit, i.e. for 36 of every 128 masks.
    l, f = 8, 3
    r = np.arange(256, dtype=np.int64)
    x = np.full(256, 100, dtype=np.int64)

    def split(v):
        return np.stack([(v - 5) % 256, np.full(v.size, 5)]).astype(np.uint64)
    out = oracle.trunc(split(x), split(r), split((r >> f) & 15), split(r >> 7), f, l=l)
    got = out.sum(axis=0, dtype=np.uint64).astype(np.int64) % 256
    err = (got - (100 >> 3)) % 256
    wrong = ~np.isin(err, [0, 1])
    assert wrong.sum() == 72
    assert (wrong == ((36 + (r % 128)) >= 128)).all()
    assert set(err[wrong].tolist()) <= {(256 - 32) % 256, (256 - 32 + 1) % 256}


def test_local_shift_fails_at_the_rate_the_paper_quotes():
    # Section 4.4: with l = 64 and precision 26, a product (a value of about 2^52) is mis-truncated by
    # the two-party local shift with probability up to 2^-11 (SecureML's bound 2^(l_x+1-l) for
    # |x| < 2^l_x), and the probability grows in proportion to |x|.
    rng = np.random.default_rng(100)
    L, f = 1 << 20, 26

    def failure_rate(log_mag, seed):
        x = (rng.integers(0, 2, size=L, dtype=np.int64) * 2 - 1) * (np.int64(1) << log_mag)
        X = oracle.share(x.view(np.uint64), 2, seed, oracle.STREAM_X)
        got = oracle.local_shift_trunc(X, f).sum(axis=0, dtype=np.uint64).view(np.int64)
        return (np.abs(got - (x >> f)) > 1).mean()
    r52, r54 = failure_rate(52, 101), failure_rate(54, 103)
    assert 2.0 ** -13 < r52 <= 2.0 ** -11
    assert 3.0 < r54 / r52 < 5.0
    # three parties: essentially always wrong (the same paragraph, citing ABY3)
    x = np.full(4096, 1 << 52, dtype=np.int64)
    X3 = oracle.share(x.view(np.uint64), 3, 102, oracle.STREAM_X)
    got3 = oracle.local_shift_trunc(X3, f).sum(axis=0, dtype=np.uint64).view(np.int64)
    assert (np.abs(got3 - (x >> f)) > 1).mean() > 0.3


# --------------------------------------------------------------------------- fixed-point product end to end
@pytest.mark.parametrize("n,dist", [(3, "u1"), (2, "n1"), (5, "u4")])
def test_decoded_truncated_product_matches_float64(n, dist):
    rng = np.random.default_rng(110 + n)
    M, N, K, f = 24, 20, 96, 16
    draw = {"u1": lambda s: rng.uniform(-1, 1, s), "n1": lambda s: rng.normal(0, 1, s),
            "u4": lambda s: rng.uniform(-4, 4, s)}[dist]
    x, y = draw((1, M, K)), draw((1, K, N))
    X = oracle.share(oracle.encode(x, f), n, 111, oracle.STREAM_X)
    Y = oracle.share(oracle.encode(y, f), n, 111, oracle.STREAM_Y)
    A, B, C = oracle.dealer_matmul(n, 1, M, N, K, seed=111)
    Z = oracle.beaver_matmul(X, Y, A, B, C)                       # precision 2f (Section 4.3)
    r, rt, rm = oracle.trunc_dealer(n, M * N, f, seed=111)
    T = oracle.trunc(Z.reshape(n, -1), r, rt, rm, f)              # back to precision f
    got = oracle.decode(oracle.open_(T), f).reshape(M, N)
    # against the product of the values the encodings actually stand for: exact up to floor and v
    xq, yq = oracle.decode(oracle.encode(x, f), f), oracle.decode(oracle.encode(y, f), f)
    assert np.abs(got - xq[0] @ yq[0]).max() <= 2.0 * 2.0 ** -f + 1e-12
    # against the product of the original reals: the stated bound 2^-f (K+2)
    assert np.abs(got - x[0] @ y[0]).max() <= 2.0 ** -f * (K + 2)
    # before truncation the product is exact at precision 2f
    assert np.abs(oracle.decode(oracle.open_(Z), 2 * f)[0] - xq[0] @ yq[0]).max() < 1e-9


# ----------------------------------------------------------------------------- tiled batch multiplication (Section 7.3)
def test_tiled_multiplication_reconstructs_and_matches_python_integers():
    rng = np.random.default_rng(73)
    for over_inner in (True, False):
        n, outer, mid, inner = 3, 2, 5, 4
        small = outer * (mid if over_inner else inner)
        x = rng.integers(0, 1 << 64, size=small, dtype=np.uint64)
        y = rng.integers(0, 1 << 64, size=outer * mid * inner, dtype=np.uint64)
        X, Y = oracle.share(x, n, 1, oracle.STREAM_X), oracle.share(y, n, 1, oracle.STREAM_Y)
        a, b, c = oracle.dealer_mul_bcast(n, outer, mid, inner, over_inner, seed=2)
        # the triple: c opens to (tiled a) * b, in Python integers
        ao, bo, co = oracle.open_(a), oracle.open_(b), oracle.open_(c)
        z = oracle.open_(oracle.beaver_mul_bcast(X, Y, a, b, c, outer, mid, inner, over_inner))
        for o in range(outer):
            for m in range(mid):
                for i in range(inner):
                    k = (o * mid + m) * inner + i
                    s = o * mid + m if over_inner else o * inner + i
                    assert int(co[k]) == int(ao[s]) * int(bo[k]) % (1 << 64)
                    assert int(z[k]) == int(x[s]) * int(y[k]) % (1 << 64)


def test_tiling_a_factor_of_full_size_is_the_plain_multiplication():
    # inner = 1 (rows) or mid = 1 (columns): nothing is repeated, and the result is Mul itself
    rng = np.random.default_rng(74)
    n, count = 2, 50
    X, Y = rng.integers(0, 1 << 64, size=(2, n, count), dtype=np.uint64)
    a, b, c = oracle.dealer_mul(n, count, seed=3)
    want = oracle.beaver_mul(X, Y, a, b, c)
    assert (oracle.beaver_mul_bcast(X, Y, a, b, c, count, 1, 1, True) == want).all()
    assert (oracle.beaver_mul_bcast(X, Y, a, b, c, 1, 1, count, False) == want).all()
    assert (oracle.beaver_mul_bcast(X, Y, a, b, c, 5, 10, 1, True) == want).all()
