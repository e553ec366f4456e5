/*
 * CPU oracle for the local work of additive-secret-sharing Beaver multiplication
 * and probabilistic truncation over the ring Z_{2^l} (l <= 64).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is deliberately plain and slow: straight
 * loops over uint64_t with wraparound, one statement per protocol step, in the
 * paper's order and notation.  Nothing in the GPU library links, includes or
 * calls it, and it includes nothing from the GPU library.  Only the tests, the
 * smoke check and the CPU-baseline leg of the benchmark may load it.
 *
 * Every function takes host pointers.  All share tensors are party-major:
 * T[i] is party i's share, so T has shape [n][...].  Party index 0 here is the
 * paper's party 1; it holds the residual share and adds every public term.
 *
 * Ring width: functions take `l` (bits, 1..64).  Values are kept in uint64_t;
 * because 2^l divides 2^64, ordinary wraparound arithmetic followed by a mask
 * to l bits is arithmetic in Z_{2^l}.  l = 64 is the production ring; small l
 * exists so the tests can brute-force the whole ring.
 *
 * Parity pins (tests/test_oracle_pins.py): none of the functions below is
 * "parity unpinned" -- each is held by an exhaustive brute force on a tiny
 * ring, a closed form, or a Python big-integer re-computation.
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>

typedef uint64_t u64;

static inline u64 ring_mask(int l) { return l >= 64 ? ~(u64)0 : (((u64)1 << l) - 1); }

/* ------------------------------------------------------------------------ */
/* Counter-based generator of the synthetic randomness (dealer masks, shares).
 * Not from the paper: the paper draws these from an OT-based offline phase
 * (Section 4.2).  The generator is a stateless integer mixer so that the GPU
 * side can produce the same values from the same written specification:
 *
 *   mix(z)        : z ^= z>>30; z *= 0xBF58476D1CE4E5B9; z ^= z>>27;
 *                   z *= 0x94D049BB133111EB; z ^= z>>31          (SplitMix64 finaliser)
 *   absorb(h, v)  = mix(h + (v+1) * 0x9E3779B97F4A7C15)
 *   key           = absorb(absorb(absorb(0, seed), stream), party)
 *   rand64(idx)   = absorb(key, idx)
 */
static inline u64 mix64(u64 z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}
static inline u64 absorb(u64 h, u64 v) { return mix64(h + (v + 1) * 0x9E3779B97F4A7C15ull); }

u64 oracle_rand64(u64 seed, u64 stream, u64 party, u64 idx)
{
    u64 key = absorb(absorb(absorb(0, seed), stream), party);
    return absorb(key, idx);
}

/* ------------------------------------------------------------------------ */
/* Fixed-point encoding, Section 4.1 (Notations): a real x becomes the signed
 * integer floor(2^p x), held in the ring as its two's-complement residue. */
void oracle_encode(const double *x, size_t count, int p, int l, u64 *out)
{
    for (size_t k = 0; k < count; ++k) {
        double scaled = floor(ldexp(x[k], p));
        out[k] = (u64)(int64_t)scaled & ring_mask(l);
    }
}

/* Inverse map: the ring element is read as a signed integer in
 * [-2^(l-1), 2^(l-1)-1] (Section 4.1) and divided by 2^p. */
void oracle_decode(const u64 *u, size_t count, int p, int l, double *out)
{
    for (size_t k = 0; k < count; ++k) {
        u64 v = u[k] & ring_mask(l);
        int64_t s;
        if (l < 64 && (v >> (l - 1)) & 1) s = (int64_t)(v | ~ring_mask(l));
        else s = (int64_t)v;
        out[k] = ldexp((double)s, -p);
    }
}

/* ------------------------------------------------------------------------ */
/* n-out-of-n arithmetic sharing, Section 4.1: x = sum_i x_i.  Parties 1..n-1
 * take generator output, party 0 the residual. */
void oracle_share(const u64 *x, size_t count, int n, int l, u64 seed, u64 stream, u64 *shares)
{
    u64 mask = ring_mask(l);
    for (size_t k = 0; k < count; ++k) {
        u64 rest = 0;
        for (int i = 1; i < n; ++i) {
            u64 s = oracle_rand64(seed, stream, (u64)i, k) & mask;
            shares[(size_t)i * count + k] = s;
            rest += s;
        }
        shares[k] = (x[k] - rest) & mask;
    }
}

/* Opening: every party publishes its (optionally masked) share and all add
 * them up, out = sum_i (shares_i - mask_i).  With mask == NULL it is plain
 * reconstruction (Section 4.1); with the triple's A as mask it is the E = X-A
 * opening of the multiplication (Section 4.3, Multiplication). */
void oracle_open(const u64 *shares, const u64 *mask_sh, size_t count, int n, int l, u64 *out)
{
    u64 mask = ring_mask(l);
    for (size_t k = 0; k < count; ++k) {
        u64 acc = 0;
        for (int i = 0; i < n; ++i) {
            u64 v = shares[(size_t)i * count + k];
            if (mask_sh) v -= mask_sh[(size_t)i * count + k];
            acc += v;
        }
        out[k] = acc & mask;
    }
}

/* ------------------------------------------------------------------------ */
/* Plain ring matrix product, the textbook definition:
 * out[m][q] = sum_k P[m][k] * Q[k][q]  (mod 2^l), row-major.
 * The sum over k is taken for one row m at a time into that row of `out`
 * (loop order m, k, q).  Ring addition is associative and commutative, so the
 * order of the k terms cannot change a single bit. */
void oracle_ring_matmul(const u64 *P, const u64 *Q, int M, int N, int K, int l, u64 *out)
{
    u64 mask = ring_mask(l);
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        u64 *row = out + (size_t)m * N;
        for (int q = 0; q < N; ++q) row[q] = 0;
        for (int k = 0; k < K; ++k) {
            u64 p = P[(size_t)m * K + k];
            const u64 *qrow = Q + (size_t)k * N;
            for (int q = 0; q < N; ++q) row[q] += p * qrow[q];
        }
        for (int q = 0; q < N; ++q) row[q] &= mask;
    }
}

/* ------------------------------------------------------------------------ */
/* Trusted-dealer stand-in for the offline phase (Section 4.2): Beaver triples.
 * Every party's A_i and B_i is generator output; A = sum A_i, B = sum B_i;
 * C = A.B (matrix product per batch entry); C is then shared like any value.
 * Streams: sA, sB for the operand shares, sC for the C mask.
 * Shapes: A [n][batch][M][K], B [n][batch][K][N], C [n][batch][M][N]. */
void oracle_dealer_matmul(int n, int batch, int M, int N, int K, int l, u64 seed,
                          u64 sA, u64 sB, u64 sC, u64 *A, u64 *B, u64 *C,
                          u64 *scratchA, u64 *scratchB, u64 *scratchC)
{
    u64 mask = ring_mask(l);
    size_t szA = (size_t)batch * M * K, szB = (size_t)batch * K * N, szC = (size_t)batch * M * N;
    for (int i = 0; i < n; ++i) {
        for (size_t k = 0; k < szA; ++k) A[i * szA + k] = oracle_rand64(seed, sA, (u64)i, k) & mask;
        for (size_t k = 0; k < szB; ++k) B[i * szB + k] = oracle_rand64(seed, sB, (u64)i, k) & mask;
    }
    oracle_open(A, NULL, szA, n, l, scratchA);
    oracle_open(B, NULL, szB, n, l, scratchB);
    for (int b = 0; b < batch; ++b)
        oracle_ring_matmul(scratchA + (size_t)b * M * K, scratchB + (size_t)b * K * N, M, N, K, l,
                           scratchC + (size_t)b * M * N);
    oracle_share(scratchC, szC, n, l, seed, sC, C);
}

/* Elementwise triples: c = a*b per element. */
void oracle_dealer_mul(int n, size_t count, int l, u64 seed, u64 sA, u64 sB, u64 sC,
                       u64 *a, u64 *b, u64 *c, u64 *scratch)
{
    u64 mask = ring_mask(l);
    for (int i = 0; i < n; ++i)
        for (size_t k = 0; k < count; ++k) {
            a[i * count + k] = oracle_rand64(seed, sA, (u64)i, k) & mask;
            b[i * count + k] = oracle_rand64(seed, sB, (u64)i, k) & mask;
        }
    for (size_t k = 0; k < count; ++k) {
        u64 av = 0, bv = 0;
        for (int i = 0; i < n; ++i) { av += a[i * count + k]; bv += b[i * count + k]; }
        scratch[k] = (av * bv) & mask;
    }
    oracle_share(scratch, count, n, l, seed, sC, c);
}

/* ------------------------------------------------------------------------ */
/* Online phase of Mul for matrices (Section 4.3, Multiplication, with a matrix
 * triple as its last sentence says).  Steps, for each batch entry:
 *   1. every party masks its shares and all open  E = X - A,  F = Y - B;
 *   2. X.Y = (E+A).(F+B) = E.F + E.B + A.F + A.B, so party i sets
 *        Z_i = C_i + E.B_i + A_i.F      and party 0 also adds the public E.F.
 * E multiplies from the left and F from the right: matrices do not commute.
 * E_out / F_out (shape [batch][M][K], [batch][K][N]) receive the opened values.
 * If rows != NULL only the listed output rows (n_rows of them, the same row set
 * for every party and batch entry) are computed, into Z laid out
 * [n][batch][n_rows][N]; otherwise all M rows, Z [n][batch][M][N]. */
void oracle_beaver_matmul(int n, int batch, int M, int N, int K, int l,
                          const u64 *X, const u64 *Y, const u64 *A, const u64 *B, const u64 *C,
                          u64 *Z, u64 *E_out, u64 *F_out, const int *rows, int n_rows)
{
    u64 mask = ring_mask(l);
    size_t szA = (size_t)batch * M * K, szB = (size_t)batch * K * N;
    int R = rows ? n_rows : M;

    oracle_open(X, A, szA, n, l, E_out);
    oracle_open(Y, B, szB, n, l, F_out);

    for (int i = 0; i < n; ++i)
        for (int b = 0; b < batch; ++b) {
            const u64 *E = E_out + (size_t)b * M * K, *F = F_out + (size_t)b * K * N;
            const u64 *Ai = A + ((size_t)i * batch + b) * M * K;
            const u64 *Bi = B + ((size_t)i * batch + b) * K * N;
            const u64 *Ci = C + ((size_t)i * batch + b) * M * N;
            u64 *Zi = Z + ((size_t)i * batch + b) * R * N;
#pragma omp parallel for schedule(static)
            for (int rr = 0; rr < R; ++rr) {
                int m = rows ? rows[rr] : rr;
                u64 *z = Zi + (size_t)rr * N;
                for (int q = 0; q < N; ++q) z[q] = Ci[(size_t)m * N + q];
                for (int k = 0; k < K; ++k) {                    /* + E.B_i */
                    u64 e = E[(size_t)m * K + k];
                    for (int q = 0; q < N; ++q) z[q] += e * Bi[(size_t)k * N + q];
                }
                for (int k = 0; k < K; ++k) {                    /* + A_i.F */
                    u64 a = Ai[(size_t)m * K + k];
                    for (int q = 0; q < N; ++q) z[q] += a * F[(size_t)k * N + q];
                }
                if (i == 0)
                    for (int k = 0; k < K; ++k) {                /* + E.F, once */
                        u64 e = E[(size_t)m * K + k];
                        for (int q = 0; q < N; ++q) z[q] += e * F[(size_t)k * N + q];
                    }
                for (int q = 0; q < N; ++q) z[q] &= mask;
            }
        }
}

/* Online phase of Mul for arrays, elementwise (Section 4.3; the "batch
 * multiplication" of Section 7.3).  Same identity with scalar products. */
void oracle_beaver_mul(int n, size_t count, int l,
                       const u64 *x, const u64 *y, const u64 *a, const u64 *b, const u64 *c, u64 *z)
{
    u64 mask = ring_mask(l);
    for (size_t k = 0; k < count; ++k) {
        u64 e = 0, f = 0;
        for (int i = 0; i < n; ++i) {
            e += x[i * count + k] - a[i * count + k];
            f += y[i * count + k] - b[i * count + k];
        }
        for (int i = 0; i < n; ++i) {
            u64 v = c[i * count + k] + e * b[i * count + k] + a[i * count + k] * f;
            if (i == 0) v += e * f;
            z[i * count + k] = v & mask;
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Dealer tuple for truncation by f bits in Z_{2^l}: one random ring element r
 * per value (its l bits are the shared random bits), together with sharings of
 *   r_top = bits f .. l-2 of r   (an (l-1-f)-bit number), and
 *   r_msb = bit l-1 of r.
 * Streams sR, sT, sM mask the three sharings. */
void oracle_trunc_dealer(int n, size_t count, int l, int f, u64 seed, u64 sR, u64 sT, u64 sM,
                         u64 *r_sh, u64 *rtop_sh, u64 *rmsb_sh, u64 *scratch)
{
    u64 mask = ring_mask(l);
    u64 topmask = ring_mask(l - 1 - f);
    /* r itself: every party's share is generator output, r is their sum. */
    for (int i = 0; i < n; ++i)
        for (size_t k = 0; k < count; ++k)
            r_sh[i * count + k] = oracle_rand64(seed, sR, (u64)i, k) & mask;
    oracle_open(r_sh, NULL, count, n, l, scratch);              /* scratch = r */
    /* share r_top and r_msb */
    for (size_t k = 0; k < count; ++k) {
        u64 r = scratch[k];
        u64 top = (r >> f) & topmask, msb = (r >> (l - 1)) & 1;
        u64 rest_t = 0, rest_m = 0;
        for (int i = 1; i < n; ++i) {
            u64 t = oracle_rand64(seed, sT, (u64)i, k) & mask;
            u64 m = oracle_rand64(seed, sM, (u64)i, k) & mask;
            rtop_sh[i * count + k] = t; rest_t += t;
            rmsb_sh[i * count + k] = m; rest_m += m;
        }
        rtop_sh[k] = (top - rest_t) & mask;
        rmsb_sh[k] = (msb - rest_m) & mask;
    }
}

/* Signed probabilistic truncation, Section 4.4 (Truncation):
 *   Truncate(x, f) = UnsignedTruncate(x + 2^(l-2), l, f) - 2^(l-f-2),
 * valid for x in [-2^(l-2), 2^(l-2)-1].  UnsignedTruncate is the mask-and-open
 * protocol for values whose top bit is zero:
 *   1. x' = x + 2^(l-2)                      (party 0 adds the constant)
 *   2. open c = x' + r                       (r from the dealer tuple)
 *   3. c_msb = bit l-1 of c,  c' = bits f..l-2 of c
 *   4. the addition x'+r (without r's top bit) carried out of bit l-2 exactly
 *      when  r_msb XOR c_msb = 1;  as an arithmetic sharing
 *         b_i = r_msb_i + [i=0] c_msb - 2 c_msb r_msb_i
 *   5. y_i = [i=0] c' - r_top_i + 2^(l-1-f) b_i
 *   6. out_i = y_i - [i=0] 2^(l-f-2)
 * The opened result is floor(x / 2^f) + v with v in {0,1}: v is the carry of
 * the low f bits of x' and r. */
void oracle_trunc(int n, size_t count, int l, int f,
                  const u64 *x, const u64 *r, const u64 *r_top, const u64 *r_msb, u64 *out)
{
    u64 mask = ring_mask(l);
    u64 topmask = ring_mask(l - 1 - f);
    u64 bias = (u64)1 << (l - 2);
    for (size_t k = 0; k < count; ++k) {
        u64 c = bias;
        for (int i = 0; i < n; ++i) c += x[i * count + k] + r[i * count + k];
        c &= mask;
        u64 c_msb = (c >> (l - 1)) & 1;
        u64 c_top = (c >> f) & topmask;
        for (int i = 0; i < n; ++i) {
            u64 rm = r_msb[i * count + k];
            u64 b = rm - 2 * c_msb * rm;
            if (i == 0) b += c_msb;
            u64 y = ((u64)1 << (l - 1 - f)) * b - r_top[i * count + k];
            if (i == 0) y += c_top;
            if (i == 0) y -= (u64)1 << (l - f - 2);
            out[i * count + k] = y & mask;
        }
    }
}

/* Local-shift truncation of Section 4.4's second paragraph (each party shifts
 * its own share; party 0 shifts x_0, the others shift the negation and negate
 * back).  Kept only for the negative tests: it is wrong with probability
 * proportional to |x| for two parties and useless for three. */
void oracle_local_shift_trunc(int n, size_t count, int f, const u64 *x, u64 *out)
{
    for (size_t k = 0; k < count; ++k)
        for (int i = 0; i < n; ++i) {
            u64 v = x[i * count + k];
            out[i * count + k] = (i == 0) ? (v >> f) : (u64)0 - (((u64)0 - v) >> f);
        }
}

/* Number of threads the row loops actually run on, and a way to fix it (for the benchmark report's
 * all-cores and single-core figures). */
#ifdef _OPENMP
#include <omp.h>
int oracle_threads(void) { return omp_get_max_threads(); }
void oracle_set_threads(int t) { if (t >= 1) omp_set_num_threads(t); }
#else
int oracle_threads(void) { return 1; }
void oracle_set_threads(int t) { (void)t; }
#endif

/* One generator step, exposed so the tests can hold it against the published
 * SplitMix64 sequences: absorb(h, v) is output number v of SplitMix64 started
 * from state h. */
u64 oracle_absorb(u64 h, u64 v) { return absorb(h, v); }

/* out[k] = rand64(seed, stream, party, first + k): a whole generator stream at once. */
void oracle_random(u64 *out, size_t count, u64 seed, u64 stream, u64 party, u64 first)
{
    for (size_t k = 0; k < count; ++k) out[k] = oracle_rand64(seed, stream, party, first + k);
}

/* ------------------------------------------------------------------------ */
/* Local linear combination with public coefficients (Section 4.3: Addition is
 * share-wise, Scaling multiplies every share by the public k; a public
 * constant is added by party 0 only):
 *   out_i = sum_j coef[j] * in[j]_i  +  [i = 0] constant.
 * in: `terms` pointers to [n][count] share tensors. */
void oracle_lincomb(int n, size_t count, int l, int terms, const u64 *const *in, const u64 *coef,
                    u64 constant, u64 *out)
{
    u64 mask = ring_mask(l);
    for (int i = 0; i < n; ++i)
        for (size_t k = 0; k < count; ++k) {
            u64 acc = (i == 0) ? constant : 0;
            for (int j = 0; j < terms; ++j) acc += coef[j] * in[j][(size_t)i * count + k];
            out[(size_t)i * count + k] = acc & mask;
        }
}

/* ------------------------------------------------------------------------ */
/* Binary sharing (Section 4.1): a bit x is split into n bits with x = XOR_i x_i.
 * Words carry 64 independent bit positions.  Parties 1..n-1 take generator
 * output, party 0 the residual. */
void oracle_bshare(const u64 *x, size_t count, int n, u64 seed, u64 stream, u64 *shares)
{
    for (size_t k = 0; k < count; ++k) {
        u64 rest = x[k];
        for (int i = 1; i < n; ++i) {
            u64 s = oracle_rand64(seed, stream, (u64)i, k);
            shares[(size_t)i * count + k] = s;
            rest ^= s;
        }
        shares[k] = rest;
    }
}

/* Opening of a binary sharing: out = XOR_i (shares_i XOR mask_i); mask may be NULL. */
void oracle_bopen(const u64 *shares, const u64 *mask_sh, size_t count, int n, u64 *out)
{
    for (size_t k = 0; k < count; ++k) {
        u64 acc = 0;
        for (int i = 0; i < n; ++i) {
            acc ^= shares[(size_t)i * count + k];
            if (mask_sh) acc ^= mask_sh[(size_t)i * count + k];
        }
        out[k] = acc;
    }
}

/* Bit triples for AND: a_i, b_i generator output, c = (XOR a_i) AND (XOR b_i), shared. */
void oracle_dealer_and(int n, size_t count, u64 seed, u64 sA, u64 sB, u64 sC, u64 *a, u64 *b, u64 *c, u64 *scratch)
{
    for (int i = 0; i < n; ++i)
        for (size_t k = 0; k < count; ++k) {
            a[i * count + k] = oracle_rand64(seed, sA, (u64)i, k);
            b[i * count + k] = oracle_rand64(seed, sB, (u64)i, k);
        }
    for (size_t k = 0; k < count; ++k) {
        u64 av = 0, bv = 0;
        for (int i = 0; i < n; ++i) { av ^= a[i * count + k]; bv ^= b[i * count + k]; }
        scratch[k] = av & bv;
    }
    oracle_bshare(scratch, count, n, seed, sC, c);
}

/* AND of two binary sharings with a bit triple: the GF(2) form of the Beaver
 * update (XOR for addition, Section 4.3 Addition; AND for multiplication):
 *   e = XOR_i (x_i ^ a_i), f = XOR_i (y_i ^ b_i) opened,
 *   z_i = c_i ^ (e & b_i) ^ (a_i & f), and party 0 also XORs in e & f. */
void oracle_beaver_and(int n, size_t count, const u64 *x, const u64 *y, const u64 *a, const u64 *b,
                       const u64 *c, u64 *z)
{
    for (size_t k = 0; k < count; ++k) {
        u64 e = 0, f = 0;
        for (int i = 0; i < n; ++i) {
            e ^= x[i * count + k] ^ a[i * count + k];
            f ^= y[i * count + k] ^ b[i * count + k];
        }
        for (int i = 0; i < n; ++i) {
            u64 v = c[i * count + k] ^ (e & b[i * count + k]) ^ (a[i * count + k] & f);
            if (i == 0) v ^= e & f;
            z[i * count + k] = v;
        }
    }
}
