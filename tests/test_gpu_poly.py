"""GPU-vs-oracle parity of the public-coefficient linear combination with fused truncation and of the two
polynomial evaluations built on it (Section 4.4 Polynomial evaluation; Section 7.2 Eq. (4))."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2402_02320_amd import poly, spin

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).cuda()


def host(t):
    return t.cpu().numpy().view(np.uint64)


def f1_table():
    t = {}
    for ln in open(os.path.join(GOLDEN, "poly_coefficients.txt")):
        if not ln.startswith("#") and ln.strip():
            name, f1, _ = ln.split()
            t[name] = float(f1)
    return t


@pytest.mark.parametrize("n", [1, 2, 3, 5, 8])
@pytest.mark.parametrize("terms", [1, 2, 4, 8])
@pytest.mark.parametrize("count,f", [(1, 0), (1000, 0), (777, 16), (70001, 22), (4096, 1)])
def test_lincomb_trunc(n, terms, count, f):
    rng = np.random.default_rng(n * 1000 + terms * 10 + f)
    # small magnitudes so that the combination stays inside the truncation's admissible range
    xs = [rng.integers(-(1 << 40), 1 << 40, size=count, dtype=np.int64) for _ in range(terms)]
    X = [oracle.share(x.view(np.uint64), n, 3 + j, oracle.STREAM_X) for j, x in enumerate(xs)]
    coefs = [int(c) for c in rng.integers(-(1 << 16), 1 << 16, size=terms)]
    const = int(rng.integers(-(1 << 50), 1 << 50))
    want = oracle.lincomb(X, coefs, const)
    tup = None
    if f:
        r, rt, rm = oracle.trunc_dealer(n, count, f, seed=5)
        want = oracle.trunc(want, r, rt, rm, f)
        tup = (dev(r), dev(rt), dev(rm))
    got = spin.lincomb_trunc([dev(x) for x in X], coefs, const, f, tup)
    assert (host(got) == want).all()


def deal(n, count, p, seed, mul_steps, trunc_steps):
    triples = [tuple(dev(t) for t in oracle.dealer_mul(n, count, s)) for s in mul_steps]
    tuples = [tuple(dev(t) for t in oracle.trunc_dealer(n, count, f, s)) for s, f in trunc_steps]
    return triples, tuples


@pytest.mark.parametrize("n,count", [(3, 4001), (2, 1 << 16)])
def test_evaluate_poly_f1(n, count):
    t = f1_table()
    k = [t["k%d" % i] for i in range(5)]
    p, seed = 16, 9
    z = np.random.default_rng(count).uniform(0, 1, size=count)
    X = oracle.share(oracle.encode(z, p), n, 5, 1)
    want = oracle.evaluate_poly(X, k, p, seed=seed)
    # the oracle deals the power x^i from seed + 10 i (triple) and seed + 10 i + 1 (tuple), the last tuple from seed + 1
    triples, tuples = deal(n, count, p, seed, [seed + 10 * i for i in (2, 3, 4)],
                           [(seed + 10 * i + 1, p) for i in (2, 3, 4)] + [(seed + 1, p)])
    got = poly.evaluate_poly(dev(X), k, p, triples, tuples)
    assert (host(got) == want).all()
    y = oracle.decode(host(spin.open(got)), p)
    assert np.abs(y - 2.0 ** z).max() <= 2.0 ** -p * 8 + 1e-5


@pytest.mark.parametrize("n,count", [(3, 4001), (5, 1 << 16)])
def test_evaluate_completed_square_f1(n, count):
    t = f1_table()
    p, seed = 14, 13                                          # the attention block runs at precision 14 (Section 7.2)
    z = np.random.default_rng(count + 1).uniform(0, 1, size=count)
    X = oracle.share(oracle.encode(z, p), n, 6, 1)
    args = (-6, t["t3"], t["t2"], t["t1"], t["t0"], p)
    want = oracle.evaluate_completed_square(X, *args, seed=seed)
    triples, tuples = deal(n, count, p, seed, [seed + 20, seed + 22], [(seed + 21, p), (seed + 23, p + 6)])
    got = poly.evaluate_completed_square(dev(X), *args, triples, tuples)
    assert (host(got) == want).all()
    y = oracle.decode(host(spin.open(got)), p)
    assert np.abs(y * t["k4"] / t["k4p"] - 2.0 ** z).max() <= 2.0 ** -p * 8 + 1e-5
