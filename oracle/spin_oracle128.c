/*
 * CPU oracle for the same protocol steps over the ring Z_{2^128} (the paper's
 * second ring width: "64-bit or 128-bit" multiplications, Section 6; its GPU
 * kernels use __int128, Section 6.1).
 *
 * TEST INFRASTRUCTURE, like spin_oracle.c: plain loops over unsigned __int128
 * with wraparound, one statement per protocol step, no code shared with the GPU
 * library.  Every function mirrors its 64-bit namesake in spin_oracle.c; the
 * comments there carry the citations.  Ring elements are stored little-endian
 * as two uint64 words (low, high), which is the in-memory layout of
 * unsigned __int128 on x86-64.  A 128-bit generator word is the pair of
 * 64-bit generator outputs at indices 2k (low) and 2k+1 (high).
 *
 * Parity pins (tests/test_oracle_128.py): Python integers for every function,
 * the closed form of the truncation at l = 128, and agreement of the low 64
 * bits with the 64-bit oracle wherever the mathematics demands it.
 */
#include <stdint.h>
#include <stddef.h>

typedef uint64_t u64;
typedef unsigned __int128 u128;

extern u64 oracle_rand64(u64 seed, u64 stream, u64 party, u64 idx);   /* the generator of spin_oracle.c */

static inline u128 rand128(u64 seed, u64 stream, u64 party, size_t k)
{
    u128 lo = oracle_rand64(seed, stream, party, 2 * (u64)k);
    u128 hi = oracle_rand64(seed, stream, party, 2 * (u64)k + 1);
    return lo | (hi << 64);
}

/* Section 4.1: shares of parties 1..n-1 are generator output, party 0 holds the residual. */
void oracle128_share(const u128 *x, size_t count, int n, u64 seed, u64 stream, u128 *shares)
{
    for (size_t k = 0; k < count; ++k) {
        u128 rest = 0;
        for (int i = 1; i < n; ++i) {
            u128 s = rand128(seed, stream, (u64)i, k);
            shares[(size_t)i * count + k] = s;
            rest += s;
        }
        shares[k] = x[k] - rest;
    }
}

/* out = sum_i (shares_i - mask_i); mask may be NULL. */
void oracle128_open(const u128 *shares, const u128 *mask_sh, size_t count, int n, u128 *out)
{
    for (size_t k = 0; k < count; ++k) {
        u128 acc = 0;
        for (int i = 0; i < n; ++i) {
            u128 v = shares[(size_t)i * count + k];
            if (mask_sh) v -= mask_sh[(size_t)i * count + k];
            acc += v;
        }
        out[k] = acc;
    }
}

/* out[m][q] = sum_k P[m][k] Q[k][q] mod 2^128, row-major (loop order m, k, q). */
void oracle128_ring_matmul(const u128 *P, const u128 *Q, int M, int N, int K, u128 *out)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        u128 *row = out + (size_t)m * N;
        for (int q = 0; q < N; ++q) row[q] = 0;
        for (int k = 0; k < K; ++k) {
            u128 p = P[(size_t)m * K + k];
            for (int q = 0; q < N; ++q) row[q] += p * Q[(size_t)k * N + q];
        }
    }
}

/* Matrix triples: A_i, B_i generator output, C = (sum A_i).(sum B_i), shared. */
void oracle128_dealer_matmul(int n, int batch, int M, int N, int K, u64 seed, u64 sA, u64 sB, u64 sC,
                             u128 *A, u128 *B, u128 *C, u128 *scratchA, u128 *scratchB, u128 *scratchC)
{
    size_t szA = (size_t)batch * M * K, szB = (size_t)batch * K * N, szC = (size_t)batch * M * N;
    for (int i = 0; i < n; ++i) {
        for (size_t k = 0; k < szA; ++k) A[i * szA + k] = rand128(seed, sA, (u64)i, k);
        for (size_t k = 0; k < szB; ++k) B[i * szB + k] = rand128(seed, sB, (u64)i, k);
    }
    oracle128_open(A, NULL, szA, n, scratchA);
    oracle128_open(B, NULL, szB, n, scratchB);
    for (int b = 0; b < batch; ++b)
        oracle128_ring_matmul(scratchA + (size_t)b * M * K, scratchB + (size_t)b * K * N, M, N, K,
                              scratchC + (size_t)b * M * N);
    oracle128_share(scratchC, szC, n, seed, sC, C);
}

/* Elementwise triples. */
void oracle128_dealer_mul(int n, size_t count, u64 seed, u64 sA, u64 sB, u64 sC, u128 *a, u128 *b, u128 *c,
                          u128 *scratch)
{
    for (int i = 0; i < n; ++i)
        for (size_t k = 0; k < count; ++k) {
            a[i * count + k] = rand128(seed, sA, (u64)i, k);
            b[i * count + k] = rand128(seed, sB, (u64)i, k);
        }
    for (size_t k = 0; k < count; ++k) {
        u128 av = 0, bv = 0;
        for (int i = 0; i < n; ++i) { av += a[i * count + k]; bv += b[i * count + k]; }
        scratch[k] = av * bv;
    }
    oracle128_share(scratch, count, n, seed, sC, c);
}

/* Z_i = C_i + E.B_i + A_i.F, party 0 adds E.F; E = sum(X_i - A_i), F = sum(Y_i - B_i). */
void oracle128_beaver_matmul(int n, int batch, int M, int N, int K, const u128 *X, const u128 *Y,
                             const u128 *A, const u128 *B, const u128 *C, u128 *Z, u128 *E_out, u128 *F_out)
{
    size_t szA = (size_t)batch * M * K, szB = (size_t)batch * K * N;
    oracle128_open(X, A, szA, n, E_out);
    oracle128_open(Y, B, szB, n, F_out);
    for (int i = 0; i < n; ++i)
        for (int b = 0; b < batch; ++b) {
            const u128 *E = E_out + (size_t)b * M * K, *F = F_out + (size_t)b * K * N;
            const u128 *Ai = A + ((size_t)i * batch + b) * M * K;
            const u128 *Bi = B + ((size_t)i * batch + b) * K * N;
            const u128 *Ci = C + ((size_t)i * batch + b) * M * N;
            u128 *Zi = Z + ((size_t)i * batch + b) * M * N;
#pragma omp parallel for schedule(static)
            for (int m = 0; m < M; ++m) {
                u128 *z = Zi + (size_t)m * N;
                for (int q = 0; q < N; ++q) z[q] = Ci[(size_t)m * N + q];
                for (int k = 0; k < K; ++k) {                    /* + E.B_i */
                    u128 e = E[(size_t)m * K + k];
                    for (int q = 0; q < N; ++q) z[q] += e * Bi[(size_t)k * N + q];
                }
                for (int k = 0; k < K; ++k) {                    /* + A_i.F */
                    u128 a = Ai[(size_t)m * K + k];
                    for (int q = 0; q < N; ++q) z[q] += a * F[(size_t)k * N + q];
                }
                if (i == 0)
                    for (int k = 0; k < K; ++k) {                /* + E.F, once */
                        u128 e = E[(size_t)m * K + k];
                        for (int q = 0; q < N; ++q) z[q] += e * F[(size_t)k * N + q];
                    }
            }
        }
}

void oracle128_beaver_mul(int n, size_t count, const u128 *x, const u128 *y, const u128 *a, const u128 *b,
                          const u128 *c, u128 *z)
{
    for (size_t k = 0; k < count; ++k) {
        u128 e = 0, f = 0;
        for (int i = 0; i < n; ++i) {
            e += x[i * count + k] - a[i * count + k];
            f += y[i * count + k] - b[i * count + k];
        }
        for (int i = 0; i < n; ++i) {
            u128 v = c[i * count + k] + e * b[i * count + k] + a[i * count + k] * f;
            if (i == 0) v += e * f;
            z[i * count + k] = v;
        }
    }
}

/* Truncation tuple at l = 128: r, r_top = bits f..126 of r, r_msb = bit 127 of r, all shared. */
void oracle128_trunc_dealer(int n, size_t count, int f, u64 seed, u64 sR, u64 sT, u64 sM,
                            u128 *r_sh, u128 *rtop_sh, u128 *rmsb_sh, u128 *scratch)
{
    const u128 topmask = (((u128)1) << (127 - f)) - 1;
    for (int i = 0; i < n; ++i)
        for (size_t k = 0; k < count; ++k) r_sh[i * count + k] = rand128(seed, sR, (u64)i, k);
    oracle128_open(r_sh, NULL, count, n, scratch);
    for (size_t k = 0; k < count; ++k) {
        u128 r = scratch[k];
        u128 top = (r >> f) & topmask, msb = r >> 127;
        u128 rest_t = 0, rest_m = 0;
        for (int i = 1; i < n; ++i) {
            u128 t = rand128(seed, sT, (u64)i, k), m = rand128(seed, sM, (u64)i, k);
            rtop_sh[i * count + k] = t; rest_t += t;
            rmsb_sh[i * count + k] = m; rest_m += m;
        }
        rtop_sh[k] = top - rest_t;
        rmsb_sh[k] = msb - rest_m;
    }
}

/* Signed probabilistic truncation, Section 4.4, at l = 128 (steps as in oracle_trunc). */
void oracle128_trunc(int n, size_t count, int f, const u128 *x, const u128 *r, const u128 *r_top,
                     const u128 *r_msb, u128 *out)
{
    const int l = 128;
    const u128 topmask = (((u128)1) << (l - 1 - f)) - 1;
    const u128 bias = (u128)1 << (l - 2);
    for (size_t k = 0; k < count; ++k) {
        u128 c = bias;
        for (int i = 0; i < n; ++i) c += x[i * count + k] + r[i * count + k];
        u128 c_msb = c >> (l - 1);
        u128 c_top = (c >> f) & topmask;
        for (int i = 0; i < n; ++i) {
            u128 rm = r_msb[i * count + k];
            u128 b = rm - 2 * c_msb * rm;
            if (i == 0) b += c_msb;
            u128 y = ((u128)1 << (l - 1 - f)) * b - r_top[i * count + k];
            if (i == 0) y += c_top;
            if (i == 0) y -= (u128)1 << (l - f - 2);
            out[i * count + k] = y;
        }
    }
}
