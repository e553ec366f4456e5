"""Polynomial evaluation on shares with public coefficients, orchestrated over the library's kernels
(every arithmetic step runs on the GPU; this module only sequences calls and encodes the public
coefficients).

Section 4.4 (Polynomial evaluation): powers by Mul + Truncate, terms a_i x^i scaled without truncation
and summed, one truncation at the end.  Section 7.2, Eq. (4): the completed-square quartic with its
leading power-of-two factor folded into the last truncation.

Triples and truncation tuples are passed in (dealt by whoever plays the offline phase)."""
import math

from . import spin


def encode_public(v, p):
    """[v]_p = floor(v * 2^p) of one public real (Section 4.1)."""
    return math.floor(math.ldexp(v, p))


def evaluate_poly(x, coeffs, p, triples, tuples):
    """x: [n, count] shares of [x]_p.  coeffs[i] multiplies x^i.  triples[i-2] = (a, b, c) for the power
    x^i (i = 2..d); tuples[i-2] its truncation tuple; tuples[-1] the final truncation tuple."""
    d = len(coeffs) - 1
    powers = [x]
    for i in range(2, d + 1):
        a, b, c = triples[i - 2]
        powers.append(spin.beaver_mul_trunc(powers[-1], x, a, b, c, *tuples[i - 2], p))   # Mul + Truncate, one pass
    return spin.lincomb_trunc(powers, [encode_public(coeffs[i], p) for i in range(1, d + 1)],
                              encode_public(coeffs[0], 2 * p), p, tuples[-1])


def evaluate_completed_square(x, k4p_log2, t3, t2, t1, t0, p, triples, tuples):
    """f'(x) = 2^k4p_log2 ((x + t3)^2 + t2)^2 + (2^k4p_log2 t1) x + 2^k4p_log2 t0  (Section 7.2, Eq. (4)).
    triples: two (a, b, c); tuples: (tuple for truncating (x+t3)^2 by p, tuple for the last truncation by
    p - k4p_log2)."""
    shift = -k4p_log2
    k4p = 2.0 ** k4p_log2
    u = spin.lincomb_trunc([x], [1], encode_public(t3, p))
    u2 = spin.beaver_mul_trunc(u, u, *triples[0], *tuples[0], p)
    v = spin.lincomb_trunc([u2], [1], encode_public(t2, p), out=u2)
    v2 = spin.beaver_mul(v, v, *triples[1])
    return spin.lincomb_trunc([v2, x], [1, encode_public(k4p * t1, p) << shift],
                              encode_public(k4p * t0, 2 * p) << shift, p + shift, tuples[1], out=v2)
