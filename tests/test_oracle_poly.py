"""Pins of the oracle's linear combination and polynomial Evaluate (Section 4.4; Section 7.2 Eq. (4)):
big integers, exhaustive enumeration of the truncation outcomes on a 16-bit ring, and the coefficient
table the paper prints."""
import os

import numpy as np

import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def paper_coefficients():
    table = {}
    for ln in open(os.path.join(GOLDEN, "poly_coefficients.txt")):
        if ln.startswith("#") or not ln.strip():
            continue
        name, f1, f2 = ln.split()
        table[name] = (float(f1), float(f2))
    return table


def big(a):
    return np.asarray(a, dtype=np.uint64).astype(object)


def test_lincomb_against_big_integers():
    rng = np.random.default_rng(1)
    n, L = 3, 200
    terms = [rng.integers(0, 1 << 64, size=(n, L), dtype=np.uint64) for _ in range(4)]
    coefs = [3, (1 << 64) - 5, 0x123456789ABCDEF, 1]
    const = 0xDEADBEEF12345
    got = oracle.lincomb(terms, coefs, const)
    for i in range(n):
        want = (sum(c * big(t[i]) for c, t in zip(coefs, terms)) + (const if i == 0 else 0)) % (1 << 64)
        assert (big(got[i]) == want).all()
    # opened: the combination of the opened values plus the constant, once
    opened = sum(c * big(oracle.open_(t)) for c, t in zip(coefs, terms)) + const
    assert (big(oracle.open_(got)) == opened % (1 << 64)).all()
    # one term, coefficient 1, no constant: identity
    assert (oracle.lincomb([terms[0]], [1]) == terms[0]).all()


def test_printed_completed_square_coefficients_reproduce_the_quartic():
    # k4 (((z+t3)^2 + t2)^2 + t1 z + t0) expanded must give back k3..k0 (Section 7.2, Eq. (1)-(2))
    t = paper_coefficients()
    for col in (0, 1):
        k4, k3, k2, k1, k0 = (t[k][col] for k in ("k4", "k3", "k2", "k1", "k0"))
        t3, t2, t1, t0 = (t[k][col] for k in ("t3", "t2", "t1", "t0"))
        if col == 1:
            # The table's t1 for f2 (-0.366125013) does not reproduce k1 = 1.442547; ten times it does, so the
            # printed decimal point is taken to be misplaced.  f2 (the logarithm's polynomial) is not used here.
            assert abs(k4 * (4 * t3 ** 3 + 4 * t3 * t2 + t1) - k1) > 0.5
            t1 *= 10
        assert abs(k4 * 4 * t3 - k3) < 2e-6
        assert abs(k4 * (6 * t3 ** 2 + 2 * t2) - k2) < 2e-6
        assert abs(k4 * (4 * t3 ** 3 + 4 * t3 * t2 + t1) - k1) < 2e-6
        assert abs(k4 * ((t3 ** 2 + t2) ** 2 + t0) - k0) < 2e-6
    assert t["k4p"][0] == 2.0 ** -6 and t["k4p"][1] == -(2.0 ** -2)
    # f1 approximates 2^z on [0, 1] (Section 5.2): the Remez error of a quartic is a few 1e-6
    z = np.linspace(0, 1, 2001)
    f1 = sum(t["k%d" % i][0] * z ** i for i in range(5))
    assert np.abs(f1 - 2.0 ** z).max() < 1e-5


def possible_truncations(values, f):
    """All outcomes the probabilistic truncation allows for each exact value: floor and floor + 1."""
    out = set()
    for v in values:
        out.add(v >> f)
        out.add((v >> f) + 1)
    return out


def test_evaluate_poly_exhaustive_on_a_16_bit_ring():
    # l = 16, p = 4, quadratic with public coefficients; every admissible x in [-2, 2).  The opened result
    # must be one of the values that follow from floor-or-floor+1 at each of the two truncations.
    l, p, n = 16, 4, 3
    a0, a1, a2 = 0.8125, -1.375, 0.5625                     # exactly representable at precision 4
    xs = np.arange(-32, 32)
    X = oracle.share((xs % (1 << l)).astype(np.uint64), n, 7, 1, l=l)
    got = oracle.open_(oracle.evaluate_poly(X, [a0, a1, a2], p, seed=11, l=l), l=l).astype(np.int64)
    got = np.where(got >= 1 << (l - 1), got - (1 << l), got)
    A0, A1, A2 = int(a0 * 2 ** (2 * p)), int(a1 * 2 ** p), int(a2 * 2 ** p)
    for x, g in zip(xs, got):
        squares = possible_truncations([int(x) * int(x)], p)
        sums = [A2 * s + A1 * int(x) + A0 for s in squares]
        assert int(g) in possible_truncations(sums, p), (x, g)


def test_evaluate_poly_follows_the_float_polynomial():
    t = paper_coefficients()
    k = [t["k%d" % i][0] for i in range(5)]
    p, n = 16, 3
    z = np.linspace(0, 1, 4001)
    X = oracle.share(oracle.encode(z, p), n, 5, 1)
    y = oracle.decode(oracle.open_(oracle.evaluate_poly(X, k, p, seed=9)), p)
    # each of the three power truncations and the final one is off by at most one unit, scaled by |a_i|
    bound = 2.0 ** -p * (2 + sum(abs(c) * (i + 1) for i, c in enumerate(k)))
    assert np.abs(y - np.polyval(k[::-1], z)).max() <= bound
    assert np.abs(y - 2.0 ** z).max() <= bound + 1e-5


def test_completed_square_matches_the_rescaled_quartic():
    t = paper_coefficients()
    p, n = 16, 2
    z = np.linspace(0, 1, 4001)
    X = oracle.share(oracle.encode(z, p), n, 6, 1)
    y = oracle.decode(oracle.open_(oracle.evaluate_completed_square(
        X, -6, t["t3"][0], t["t2"][0], t["t1"][0], t["t0"][0], p, seed=13)), p)
    want = t["k4p"][0] * (((z + t["t3"][0]) ** 2 + t["t2"][0]) ** 2 + t["t1"][0] * z + t["t0"][0])
    assert np.abs(y - want).max() <= 2.0 ** -p * 8
    # up to the common factor k4'/k4 this is f1, i.e. 2^z (the factor cancels in Softmax, Section 7.2)
    assert np.abs(y * t["k4"][0] / t["k4p"][0] - 2.0 ** z).max() <= 2.0 ** -p * 8 + 1e-5


def test_completed_square_exhaustive_on_a_20_bit_ring():
    # l = 20, p = 4, k4' = 2^-2: enumerate the floor-or-floor+1 outcomes of the two truncations
    l, p, n, sh = 20, 4, 2, 2
    t3, t2, t1, t0 = 0.5, 1.25, -0.75, 2.0
    xs = np.arange(-16, 16)
    X = oracle.share((xs % (1 << l)).astype(np.uint64), n, 8, 1, l=l)
    got = oracle.open_(oracle.evaluate_completed_square(X, -sh, t3, t2, t1, t0, p, seed=17, l=l), l=l).astype(np.int64)
    got = np.where(got >= 1 << (l - 1), got - (1 << l), got)
    T3, T2 = int(t3 * 2 ** p), int(t2 * 2 ** p)
    lin, const = int(2.0 ** -sh * t1 * 2 ** p) << sh, int(2.0 ** -sh * t0 * 2 ** (2 * p)) << sh
    assert int(2.0 ** -sh * t1 * 2 ** p) == np.floor(2.0 ** -sh * t1 * 2 ** p)      # exactly representable
    for x, g in zip(xs, got):
        u = int(x) + T3
        vs = [q + T2 for q in possible_truncations([u * u], p)]
        sums = [v * v + lin * int(x) + const for v in vs]
        assert int(g) in possible_truncations(sums, p + sh), (x, g)
