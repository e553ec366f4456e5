"""ctypes front end of the CPU oracle (oracle/spin_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by __graft_entry__.smoke() and by
the cpu_baseline leg of bench.py; never by the GPU package.  All arrays are
numpy uint64 on the host, party-major ([n][...]).  The wrappers only allocate
outputs and marshal pointers; every protocol step is in the C file.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spin_oracle.c")
_SRC128 = os.path.join(_HERE, "spin_oracle128.c")
_LIB = os.path.join(_HERE, "liboracle.so")

# stream ids of the synthetic generator (which tensor a random word belongs to)
STREAM_X, STREAM_Y, STREAM_A, STREAM_B, STREAM_C = 1, 2, 3, 4, 5
STREAM_R, STREAM_RTOP, STREAM_RMSB = 6, 7, 8


def build(force=True):
    """Compile the oracle with gcc (-O2, OpenMP for the row loops)."""
    stale = not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_SRC128))
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
             "-Wall", "-Wextra", "-o", _LIB, _SRC, _SRC128, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_LIB)
        u64, sz, i32, p = ctypes.c_uint64, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p
        L.oracle_rand64.restype = u64
        L.oracle_rand64.argtypes = [u64, u64, u64, u64]
        L.oracle_absorb.restype = u64
        L.oracle_absorb.argtypes = [u64, u64]
        L.oracle_encode.argtypes = [p, sz, i32, i32, p]
        L.oracle_decode.argtypes = [p, sz, i32, i32, p]
        L.oracle_share.argtypes = [p, sz, i32, i32, u64, u64, p]
        L.oracle_open.argtypes = [p, p, sz, i32, i32, p]
        L.oracle_ring_matmul.argtypes = [p, p, i32, i32, i32, i32, p]
        L.oracle_dealer_matmul.argtypes = [i32, i32, i32, i32, i32, i32, u64, u64, u64, u64] + [p] * 6
        L.oracle_dealer_mul.argtypes = [i32, sz, i32, u64, u64, u64, u64, p, p, p, p]
        L.oracle_beaver_matmul.argtypes = [i32] * 6 + [p] * 8 + [p, i32]
        L.oracle_beaver_mul.argtypes = [i32, sz, i32] + [p] * 6
        L.oracle_trunc_dealer.argtypes = [i32, sz, i32, i32, u64, u64, u64, u64, p, p, p, p]
        L.oracle_trunc.argtypes = [i32, sz, i32, i32] + [p] * 5
        L.oracle_local_shift_trunc.argtypes = [i32, sz, i32, p, p]
        L.oracle_threads.restype = i32
        L.oracle128_share.argtypes = [p, sz, i32, u64, u64, p]
        L.oracle128_open.argtypes = [p, p, sz, i32, p]
        L.oracle128_ring_matmul.argtypes = [p, p, i32, i32, i32, p]
        L.oracle128_dealer_matmul.argtypes = [i32, i32, i32, i32, i32, u64, u64, u64, u64] + [p] * 6
        L.oracle128_dealer_mul.argtypes = [i32, sz, u64, u64, u64, u64, p, p, p, p]
        L.oracle128_beaver_matmul.argtypes = [i32] * 5 + [p] * 8
        L.oracle128_beaver_mul.argtypes = [i32, sz] + [p] * 6
        L.oracle128_trunc_dealer.argtypes = [i32, sz, i32, u64, u64, u64, u64, p, p, p, p]
        L.oracle128_trunc.argtypes = [i32, sz, i32] + [p] * 5
        for name in ("share", "open", "ring_matmul", "dealer_matmul", "dealer_mul", "beaver_matmul", "beaver_mul",
                     "trunc_dealer", "trunc"):
            getattr(L, "oracle128_" + name).restype = None
        L.oracle_bshare.argtypes = [p, sz, i32, u64, u64, p]
        L.oracle_bopen.argtypes = [p, p, sz, i32, p]
        L.oracle_dealer_and.argtypes = [i32, sz, u64, u64, u64, u64, p, p, p, p]
        L.oracle_beaver_and.argtypes = [i32, sz] + [p] * 6
        for name in ("oracle_bshare", "oracle_bopen", "oracle_dealer_and", "oracle_beaver_and"):
            getattr(L, name).restype = None
        L.oracle_lincomb.argtypes = [i32, sz, i32, i32, p, p, u64, p]
        L.oracle_lincomb.restype = None
        L.oracle_random.argtypes = [p, sz, u64, u64, u64, u64]
        L.oracle_random.restype = None
        for name in ("oracle_encode", "oracle_decode", "oracle_share", "oracle_open",
                     "oracle_ring_matmul", "oracle_dealer_matmul", "oracle_dealer_mul",
                     "oracle_beaver_matmul", "oracle_beaver_mul", "oracle_trunc_dealer",
                     "oracle_trunc", "oracle_local_shift_trunc"):
            getattr(L, name).restype = None
        _lib = L
    return _lib


def _u64(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint64:
        a = a.view(np.uint64) if a.dtype == np.int64 else a.astype(np.uint64)
    return a


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def threads():
    return int(lib().oracle_threads())


def set_threads(t):
    lib().oracle_set_threads(int(t))


def rand64(seed, stream, party, idx):
    return int(lib().oracle_rand64(seed, stream, party, idx))


def encode(x, p, l=64):
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty(x.shape, dtype=np.uint64)
    lib().oracle_encode(_ptr(x), x.size, p, l, _ptr(out))
    return out


def decode(u, p, l=64):
    u = _u64(u)
    out = np.empty(u.shape, dtype=np.float64)
    lib().oracle_decode(_ptr(u), u.size, p, l, _ptr(out))
    return out


def share(x, n, seed, stream, l=64):
    x = _u64(x)
    out = np.empty((n,) + x.shape, dtype=np.uint64)
    lib().oracle_share(_ptr(x), x.size, n, l, seed, stream, _ptr(out))
    return out


def open_(shares, mask=None, l=64):
    shares = _u64(shares)
    n = shares.shape[0]
    out = np.empty(shares.shape[1:], dtype=np.uint64)
    if mask is not None:
        mask = _u64(mask)
        assert mask.shape == shares.shape
    lib().oracle_open(_ptr(shares), _ptr(mask), out.size, n, l, _ptr(out))
    return out


def ring_matmul(P, Q, l=64):
    P, Q = _u64(P), _u64(Q)
    M, K = P.shape
    K2, N = Q.shape
    assert K == K2
    out = np.empty((M, N), dtype=np.uint64)
    lib().oracle_ring_matmul(_ptr(P), _ptr(Q), M, N, K, l, _ptr(out))
    return out


def dealer_matmul(n, batch, M, N, K, seed, l=64):
    A = np.empty((n, batch, M, K), dtype=np.uint64)
    B = np.empty((n, batch, K, N), dtype=np.uint64)
    C = np.empty((n, batch, M, N), dtype=np.uint64)
    sa = np.empty((batch, M, K), dtype=np.uint64)
    sb = np.empty((batch, K, N), dtype=np.uint64)
    sc = np.empty((batch, M, N), dtype=np.uint64)
    lib().oracle_dealer_matmul(n, batch, M, N, K, l, seed, STREAM_A, STREAM_B, STREAM_C,
                               _ptr(A), _ptr(B), _ptr(C), _ptr(sa), _ptr(sb), _ptr(sc))
    return A, B, C


def dealer_mul(n, count, seed, l=64):
    a = np.empty((n, count), dtype=np.uint64)
    b = np.empty((n, count), dtype=np.uint64)
    c = np.empty((n, count), dtype=np.uint64)
    s = np.empty((count,), dtype=np.uint64)
    lib().oracle_dealer_mul(n, count, l, seed, STREAM_A, STREAM_B, STREAM_C,
                            _ptr(a), _ptr(b), _ptr(c), _ptr(s))
    return a, b, c


def beaver_matmul(X, Y, A, B, C, l=64, rows=None, return_opened=False):
    """X,A [n][batch][M][K]; Y,B [n][batch][K][N]; C [n][batch][M][N] -> Z.

    rows: optional int array of output rows to compute (Z then has n_rows rows)."""
    X, Y, A, B, C = map(_u64, (X, Y, A, B, C))
    n, batch, M, K = X.shape
    N = Y.shape[3]
    assert Y.shape == (n, batch, K, N) and A.shape == X.shape and B.shape == Y.shape
    assert C.shape == (n, batch, M, N)
    E = np.empty((batch, M, K), dtype=np.uint64)
    F = np.empty((batch, K, N), dtype=np.uint64)
    if rows is None:
        Z = np.empty((n, batch, M, N), dtype=np.uint64)
        rp, nr = None, 0
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        assert rows.min() >= 0 and rows.max() < M
        Z = np.empty((n, batch, rows.size, N), dtype=np.uint64)
        rp, nr = _ptr(rows), rows.size
    lib().oracle_beaver_matmul(n, batch, M, N, K, l, _ptr(X), _ptr(Y), _ptr(A), _ptr(B), _ptr(C),
                               _ptr(Z), _ptr(E), _ptr(F), rp, nr)
    return (Z, E, F) if return_opened else Z


def beaver_mul(x, y, a, b, c, l=64):
    x, y, a, b, c = map(_u64, (x, y, a, b, c))
    n = x.shape[0]
    count = x[0].size
    z = np.empty(x.shape, dtype=np.uint64)
    lib().oracle_beaver_mul(n, count, l, _ptr(x), _ptr(y), _ptr(a), _ptr(b), _ptr(c), _ptr(z))
    return z


def tile_factor(x, outer, mid, inner, over_inner):
    """Section 7.3: before the batch multiplication E * R the smaller array is tiled up to the size of the
    other one ("the notation E * R implies this tiling").  x: [n][outer][mid] (over_inner, one factor per row)
    or [n][outer][inner] (one factor per column) -> [n][outer*mid*inner]."""
    x = _u64(x)
    n = x.shape[0]
    if over_inner:
        t = np.broadcast_to(x.reshape(n, outer, mid, 1), (n, outer, mid, inner))
    else:
        t = np.broadcast_to(x.reshape(n, outer, 1, inner), (n, outer, mid, inner))
    return np.ascontiguousarray(t).reshape(n, -1)


def dealer_mul_bcast(n, outer, mid, inner, over_inner, seed, l=64):
    """Triple for the tiled multiplication: a has the shape of the small factor and is tiled like it,
    b is full-sized, c shares (tiled a) * b."""
    small = outer * (mid if over_inner else inner)
    full = outer * mid * inner
    a = np.stack([random(small, seed, STREAM_A, i) for i in range(n)])
    b = np.stack([random(full, seed, STREAM_B, i) for i in range(n)])
    if l < 64:
        a &= np.uint64((1 << l) - 1)
        b &= np.uint64((1 << l) - 1)
    prod = open_(tile_factor(a, outer, mid, inner, over_inner), l=l) * open_(b, l=l)      # uint64 arithmetic wraps
    if l < 64:
        prod &= np.uint64((1 << l) - 1)
    return a, b, share(prod, n, seed, STREAM_C, l=l)


def beaver_mul_bcast(x, y, a, b, c, outer, mid, inner, over_inner, l=64):
    """The batch multiplication with one factor tiled (Section 7.3), by its definition: tile, then Mul."""
    return beaver_mul(tile_factor(x, outer, mid, inner, over_inner), y,
                      tile_factor(a, outer, mid, inner, over_inner), b, c, l=l)


def trunc_dealer(n, count, f, seed, l=64):
    r = np.empty((n, count), dtype=np.uint64)
    rt = np.empty((n, count), dtype=np.uint64)
    rm = np.empty((n, count), dtype=np.uint64)
    s = np.empty((count,), dtype=np.uint64)
    lib().oracle_trunc_dealer(n, count, l, f, seed, STREAM_R, STREAM_RTOP, STREAM_RMSB,
                              _ptr(r), _ptr(rt), _ptr(rm), _ptr(s))
    return r, rt, rm


def trunc(x, r, r_top, r_msb, f, l=64):
    x, r, r_top, r_msb = map(_u64, (x, r, r_top, r_msb))
    n = x.shape[0]
    count = x[0].size
    out = np.empty(x.shape, dtype=np.uint64)
    lib().oracle_trunc(n, count, l, f, _ptr(x), _ptr(r), _ptr(r_top), _ptr(r_msb), _ptr(out))
    return out


def local_shift_trunc(x, f):
    x = _u64(x)
    n = x.shape[0]
    out = np.empty(x.shape, dtype=np.uint64)
    lib().oracle_local_shift_trunc(n, x[0].size, f, _ptr(x), _ptr(out))
    return out


def cast_64_to_32(shares):
    """Section 7.1 (mixing bit lengths): the local Fixed64 -> Fixed32 cast.  Every party reduces its
    own share mod 2^32; the result is returned as ring-32 elements in uint64 storage, the form the
    l = 32 calls of this module take."""
    return _u64(shares) & np.uint64(0xFFFFFFFF)


def absorb(h, v):
    return int(lib().oracle_absorb(h, v))


def random(count, seed, stream, party, first=0):
    out = np.empty((count,), dtype=np.uint64)
    lib().oracle_random(_ptr(out), count, seed, stream, party, first)
    return out


def lincomb(terms, coefs, constant=0, l=64):
    """out_i = sum_j coefs[j] * terms[j]_i + [i=0] constant (Section 4.3, Addition and Scaling)."""
    terms = [_u64(t) for t in terms]
    n = terms[0].shape[0]
    count = terms[0][0].size
    assert all(t.shape == terms[0].shape for t in terms) and len(coefs) == len(terms)
    ptrs = (ctypes.c_void_p * len(terms))(*[t.ctypes.data for t in terms])
    cf = np.array([int(c) % (1 << 64) for c in coefs], dtype=np.uint64)
    out = np.empty(terms[0].shape, dtype=np.uint64)
    lib().oracle_lincomb(n, count, l, len(terms), ptrs, _ptr(cf), int(constant) % (1 << 64), _ptr(out))
    return out


def _enc1(v, p):
    """[v]_p of one public real (Section 4.1)."""
    return int(encode(np.array([v]), p)[0])


def evaluate_poly(x_sh, coeffs, p, seed, l=64):
    """Evaluate (Section 4.4, Polynomial evaluation): f(x) = sum_i coeffs[i] x^i with public coefficients.

    The powers x^2 .. x^d are formed one after the other by Mul + Truncate; the terms a_i x^i are
    scaled without truncation (precision 2p) and summed, a_0 joins at precision 2p, and a single
    Truncate brings the sum back to precision p.  Triples and truncation tuples are dealt from
    `seed + step`.  Returns shares of [f(x)]_p."""
    x_sh = _u64(x_sh)
    n = x_sh.shape[0]
    flat = x_sh.reshape(n, -1)
    count = flat.shape[1]
    d = len(coeffs) - 1
    powers = [flat]
    for i in range(2, d + 1):
        a, b, c = dealer_mul(n, count, seed + 10 * i, l)
        prod = beaver_mul(powers[-1], flat, a, b, c, l)
        r, rt, rm = trunc_dealer(n, count, p, seed + 10 * i + 1, l)
        powers.append(trunc(prod, r, rt, rm, p, l))
    total = lincomb(powers, [_enc1(coeffs[i], p) for i in range(1, d + 1)], _enc1(coeffs[0], 2 * p), l)
    r, rt, rm = trunc_dealer(n, count, p, seed + 1, l)
    return trunc(total, r, rt, rm, p, l).reshape(x_sh.shape)


def evaluate_completed_square(x_sh, k4p_log2, t3, t2, t1, t0, p, seed, l=64):
    """The completed-square evaluation of a quartic (Section 7.2, Eq. (4)):
        f'(x) = k4' ((x + t3)^2 + t2)^2 + (k4' t1) x + k4' t0,   k4' = 2^k4p_log2 (a power of two).
    Two secure multiplications; the factor k4' is not multiplied in but folded into the last
    truncation, which removes p - k4p_log2 bits instead of p; the linear and constant terms are
    pre-scaled by 2^-k4p_log2 so that they join that same truncation."""
    x_sh = _u64(x_sh)
    n = x_sh.shape[0]
    flat = x_sh.reshape(n, -1)
    count = flat.shape[1]
    shift = -k4p_log2                                   # k4' = 2^-shift
    k4p = 2.0 ** k4p_log2
    u = lincomb([flat], [1], _enc1(t3, p), l)                               # x + t3
    a, b, c = dealer_mul(n, count, seed + 20, l)
    r, rt, rm = trunc_dealer(n, count, p, seed + 21, l)
    u2 = trunc(beaver_mul(u, u, a, b, c, l), r, rt, rm, p, l)               # (x + t3)^2 at precision p
    v = lincomb([u2], [1], _enc1(t2, p), l)                                 # ... + t2
    a, b, c = dealer_mul(n, count, seed + 22, l)
    v2 = beaver_mul(v, v, a, b, c, l)                                       # precision 2p, kept
    # v^2 + 2^shift (k4' t1) x + 2^shift k4' t0, all at precision 2p, then one truncation by p + shift
    total = lincomb([v2, flat], [1, _enc1(k4p * t1, p) << shift], _enc1(k4p * t0, 2 * p) << shift, l)
    r, rt, rm = trunc_dealer(n, count, p + shift, seed + 23, l)
    return trunc(total, r, rt, rm, p + shift, l).reshape(x_sh.shape)


# ---- binary sharing (Section 4.1), 64 bit positions per word
def bshare(x, n, seed, stream):
    x = _u64(x)
    out = np.empty((n,) + x.shape, dtype=np.uint64)
    lib().oracle_bshare(_ptr(x), x.size, n, seed, stream, _ptr(out))
    return out


def bopen(shares, mask=None):
    shares = _u64(shares)
    out = np.empty(shares.shape[1:], dtype=np.uint64)
    if mask is not None:
        mask = _u64(mask)
    lib().oracle_bopen(_ptr(shares), _ptr(mask), out.size, shares.shape[0], _ptr(out))
    return out


def dealer_and(n, count, seed):
    a = np.empty((n, count), dtype=np.uint64)
    b = np.empty((n, count), dtype=np.uint64)
    c = np.empty((n, count), dtype=np.uint64)
    s = np.empty((count,), dtype=np.uint64)
    lib().oracle_dealer_and(n, count, seed, STREAM_A, STREAM_B, STREAM_C, _ptr(a), _ptr(b), _ptr(c), _ptr(s))
    return a, b, c


def beaver_and(x, y, a, b, c):
    x, y, a, b, c = map(_u64, (x, y, a, b, c))
    z = np.empty(x.shape, dtype=np.uint64)
    lib().oracle_beaver_and(x.shape[0], x[0].size, _ptr(x), _ptr(y), _ptr(a), _ptr(b), _ptr(c), _ptr(z))
    return z


# ---- ring Z_2^128: arrays carry a trailing axis of two uint64 words (low, high) ----------------------
class r128:
    """Wrappers of oracle/spin_oracle128.c.  A ring tensor of shape S is a uint64 array of shape S + (2,)."""

    @staticmethod
    def _w(a):
        a = _u64(a)
        assert a.shape[-1] == 2
        return a

    @staticmethod
    def from_ints(values, shape=None):
        flat = [int(v) % (1 << 128) for v in np.asarray(values, dtype=object).ravel()]
        out = np.array([[v & ((1 << 64) - 1), v >> 64] for v in flat], dtype=np.uint64)
        shp = np.asarray(values, dtype=object).shape if shape is None else shape
        return out.reshape(tuple(shp) + (2,))

    @staticmethod
    def to_ints(a):
        a = r128._w(a)
        lo, hi = a[..., 0].astype(object), a[..., 1].astype(object)
        return lo + hi * (1 << 64)

    @staticmethod
    def share(x, n, seed, stream):
        x = r128._w(x)
        out = np.empty((n,) + x.shape, dtype=np.uint64)
        lib().oracle128_share(_ptr(x), x.size // 2, n, seed, stream, _ptr(out))
        return out

    @staticmethod
    def open_(shares, mask=None):
        shares = r128._w(shares)
        out = np.empty(shares.shape[1:], dtype=np.uint64)
        if mask is not None:
            mask = r128._w(mask)
        lib().oracle128_open(_ptr(shares), _ptr(mask), out.size // 2, shares.shape[0], _ptr(out))
        return out

    @staticmethod
    def ring_matmul(P, Q):
        P, Q = r128._w(P), r128._w(Q)
        M, K, _ = P.shape
        N = Q.shape[1]
        out = np.empty((M, N, 2), dtype=np.uint64)
        lib().oracle128_ring_matmul(_ptr(P), _ptr(Q), M, N, K, _ptr(out))
        return out

    @staticmethod
    def dealer_matmul(n, batch, M, N, K, seed):
        A = np.empty((n, batch, M, K, 2), dtype=np.uint64)
        B = np.empty((n, batch, K, N, 2), dtype=np.uint64)
        C = np.empty((n, batch, M, N, 2), dtype=np.uint64)
        sa, sb, sc = (np.empty(t.shape[1:], dtype=np.uint64) for t in (A, B, C))
        lib().oracle128_dealer_matmul(n, batch, M, N, K, seed, STREAM_A, STREAM_B, STREAM_C,
                                      _ptr(A), _ptr(B), _ptr(C), _ptr(sa), _ptr(sb), _ptr(sc))
        return A, B, C

    @staticmethod
    def dealer_mul(n, count, seed):
        a, b, c = (np.empty((n, count, 2), dtype=np.uint64) for _ in range(3))
        s = np.empty((count, 2), dtype=np.uint64)
        lib().oracle128_dealer_mul(n, count, seed, STREAM_A, STREAM_B, STREAM_C, _ptr(a), _ptr(b), _ptr(c), _ptr(s))
        return a, b, c

    @staticmethod
    def beaver_matmul(X, Y, A, B, C):
        X, Y, A, B, C = map(r128._w, (X, Y, A, B, C))
        n, batch, M, K, _ = X.shape
        N = Y.shape[3]
        Z = np.empty((n, batch, M, N, 2), dtype=np.uint64)
        E = np.empty((batch, M, K, 2), dtype=np.uint64)
        F = np.empty((batch, K, N, 2), dtype=np.uint64)
        lib().oracle128_beaver_matmul(n, batch, M, N, K, _ptr(X), _ptr(Y), _ptr(A), _ptr(B), _ptr(C), _ptr(Z),
                                      _ptr(E), _ptr(F))
        return Z

    @staticmethod
    def beaver_mul(x, y, a, b, c):
        x, y, a, b, c = map(r128._w, (x, y, a, b, c))
        z = np.empty(x.shape, dtype=np.uint64)
        lib().oracle128_beaver_mul(x.shape[0], x[0].size // 2, _ptr(x), _ptr(y), _ptr(a), _ptr(b), _ptr(c), _ptr(z))
        return z

    @staticmethod
    def trunc_dealer(n, count, f, seed):
        r, rt, rm = (np.empty((n, count, 2), dtype=np.uint64) for _ in range(3))
        s = np.empty((count, 2), dtype=np.uint64)
        lib().oracle128_trunc_dealer(n, count, f, seed, STREAM_R, STREAM_RTOP, STREAM_RMSB,
                                     _ptr(r), _ptr(rt), _ptr(rm), _ptr(s))
        return r, rt, rm

    @staticmethod
    def trunc(x, r, r_top, r_msb, f):
        x, r, r_top, r_msb = map(r128._w, (x, r, r_top, r_msb))
        out = np.empty(x.shape, dtype=np.uint64)
        lib().oracle128_trunc(x.shape[0], x[0].size // 2, f, _ptr(x), _ptr(r), _ptr(r_top), _ptr(r_msb), _ptr(out))
        return out
