/* Host-side sanitizer target for the CPU oracle: the oracle's C sources are compiled into this program with
 * -fsanitize=address,undefined and every function is run on small heap buffers of exactly the documented size,
 * over several ring widths, party counts and ragged shapes, with and without a row subset.  An out-of-bounds
 * access, a misaligned access or undefined arithmetic in the oracle ends the run with a sanitizer report; the
 * invariants checked here (reconstruction of shares, of the Beaver product and of the truncation tuple) make sure
 * the calls did real work.  Built and run by tests/test_sanitizers.py; no GPU involved. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef uint64_t u64;
typedef unsigned __int128 u128;

u64 oracle_rand64(u64 seed, u64 stream, u64 party, u64 idx);
void oracle_random(u64 *out, size_t count, u64 seed, u64 stream, u64 party, u64 first);
void oracle_encode(const double *x, size_t count, int p, int l, u64 *out);
void oracle_decode(const u64 *u, size_t count, int p, int l, double *out);
void oracle_share(const u64 *x, size_t count, int n, int l, u64 seed, u64 stream, u64 *shares);
void oracle_open(const u64 *shares, const u64 *mask_sh, size_t count, int n, int l, u64 *out);
void oracle_ring_matmul(const u64 *P, const u64 *Q, int M, int N, int K, int l, u64 *out);
void oracle_dealer_matmul(int n, int batch, int M, int N, int K, int l, u64 seed, u64 sA, u64 sB, u64 sC, u64 *A,
                          u64 *B, u64 *C, u64 *scratchA, u64 *scratchB, u64 *scratchC);
void oracle_dealer_mul(int n, size_t count, int l, u64 seed, u64 sA, u64 sB, u64 sC, u64 *a, u64 *b, u64 *c, u64 *scratch);
void oracle_beaver_matmul(int n, int batch, int M, int N, int K, int l, const u64 *X, const u64 *Y, const u64 *A,
                          const u64 *B, const u64 *C, u64 *Z, u64 *E_out, u64 *F_out, const int *rows, int n_rows);
void oracle_beaver_mul(int n, size_t count, int l, const u64 *x, const u64 *y, const u64 *a, const u64 *b, const u64 *c,
                       u64 *z);
void oracle_trunc_dealer(int n, size_t count, int l, int f, u64 seed, u64 sR, u64 sT, u64 sM, u64 *r_sh, u64 *rtop_sh,
                         u64 *rmsb_sh, u64 *scratch);
void oracle_trunc(int n, size_t count, int l, int f, const u64 *x, const u64 *r, const u64 *r_top, const u64 *r_msb,
                  u64 *out);
void oracle_local_shift_trunc(int n, size_t count, int f, const u64 *x, u64 *out);
void oracle_bshare(const u64 *x, size_t count, int n, u64 seed, u64 stream, u64 *shares);
void oracle_bopen(const u64 *shares, const u64 *mask_sh, size_t count, int n, u64 *out);
void oracle128_share(const u128 *x, size_t count, int n, u64 seed, u64 stream, u128 *shares);
void oracle128_open(const u128 *shares, const u128 *mask_sh, size_t count, int n, u128 *out);
void oracle128_ring_matmul(const u128 *P, const u128 *Q, int M, int N, int K, u128 *out);

static int failures = 0;
#define CHECK(cond, what) do { if (!(cond)) { printf("FAILED: %s (line %d)\n", what, __LINE__); ++failures; } } while (0)

static u64 *words(size_t count) { u64 *p = (u64 *)malloc(count ? count * sizeof(u64) : 1); if (!p) abort(); return p; }
static u64 mask_of(int l) { return l == 64 ? ~(u64)0 : (((u64)1 << l) - 1); }

static void one_case(int n, int batch, int M, int N, int K, int l, int f, u64 seed)
{
    const u64 mask = mask_of(l);
    const size_t szA = (size_t)batch * M * K, szB = (size_t)batch * K * N, szC = (size_t)batch * M * N;
    u64 *x = words(szA), *y = words(szB), *back = words(szA > szC ? szA : szC);
    oracle_random(x, szA, seed, 21, 0, 0);
    oracle_random(y, szB, seed, 22, 0, 5);
    for (size_t k = 0; k < szA; ++k) x[k] &= mask;
    for (size_t k = 0; k < szB; ++k) y[k] &= mask;
    u64 *X = words(n * szA), *Y = words(n * szB), *A = words(n * szA), *B = words(n * szB), *C = words(n * szC);
    u64 *sa = words(szA), *sb = words(szB), *sc = words(szC);
    oracle_share(x, szA, n, l, seed, 1, X);
    oracle_share(y, szB, n, l, seed, 2, Y);
    oracle_open(X, NULL, szA, n, l, back);
    CHECK(memcmp(back, x, szA * sizeof(u64)) == 0, "shares of X reconstruct X");
    oracle_dealer_matmul(n, batch, M, N, K, l, seed, 3, 4, 5, A, B, C, sa, sb, sc);
    u64 *Z = words(n * szC), *E = words(szA), *F = words(szB), *plain = words(szC);
    oracle_beaver_matmul(n, batch, M, N, K, l, X, Y, A, B, C, Z, E, F, NULL, 0);
    oracle_open(Z, NULL, szC, n, l, back);
    for (int b = 0; b < batch; ++b)
        oracle_ring_matmul(x + (size_t)b * M * K, y + (size_t)b * K * N, M, N, K, l, plain + (size_t)b * M * N);
    CHECK(memcmp(back, plain, szC * sizeof(u64)) == 0, "Beaver matmul shares reconstruct X.Y");
    /* a row subset: first, last and a middle row, into a buffer of exactly n * batch * rows * N words */
    int rows[3] = {0, M / 2, M - 1};
    const int nr = M >= 3 ? 3 : 1;
    u64 *Zr = words((size_t)n * batch * nr * N);
    oracle_beaver_matmul(n, batch, M, N, K, l, X, Y, A, B, C, Zr, E, F, rows, nr);
    for (int i = 0; i < n; ++i)
        for (int b = 0; b < batch; ++b)
            for (int r = 0; r < nr; ++r)
                CHECK(memcmp(Zr + (((size_t)i * batch + b) * nr + r) * N, Z + (((size_t)i * batch + b) * M + rows[r]) * N,
                             N * sizeof(u64)) == 0, "row subset equals rows of the full result");
    /* elementwise product and truncation on the same element count */
    u64 *a = words(n * szC), *bb = words(n * szC), *c = words(n * szC), *s = words(szC), *z = words(n * szC);
    oracle_dealer_mul(n, szC, l, seed, 3, 4, 5, a, bb, c, s);
    oracle_beaver_mul(n, szC, l, Z, Z, a, bb, c, z);
    u64 *r = words(n * szC), *rt = words(n * szC), *rm = words(n * szC), *out = words(n * szC);
    oracle_trunc_dealer(n, szC, l, f, seed, 6, 7, 8, r, rt, rm, s);
    oracle_open(r, NULL, szC, n, l, back);
    oracle_open(rm, NULL, szC, n, l, plain);
    for (size_t k = 0; k < szC; ++k) CHECK(plain[k] == back[k] >> (l - 1), "r_msb opens to the top bit of r");
    /* truncate small values (inside the admissible range): shares of floor(v / 2^f) or that plus one */
    for (size_t k = 0; k < szC; ++k) plain[k] = (k * 2654435761u) & (mask >> 3);
    oracle_share(plain, szC, n, l, seed, 9, Z);
    oracle_trunc(n, szC, l, f, Z, r, rt, rm, out);
    oracle_open(out, NULL, szC, n, l, back);
    for (size_t k = 0; k < szC; ++k) CHECK(back[k] - (plain[k] >> f) <= 1, "truncation is floor or floor + 1");
    if (l == 64 && n == 2) oracle_local_shift_trunc(n, szC, f, Z, out);
    if (l == 64) {
        oracle_bshare(x, szA, n, seed, 1, X);
        oracle_bopen(X, NULL, szA, n, back);
        CHECK(memcmp(back, x, szA * sizeof(u64)) == 0, "binary shares reconstruct");
    }
    double *real = (double *)malloc(szC * sizeof(double) + 8), *dec = (double *)malloc(szC * sizeof(double) + 8);
    for (size_t k = 0; k < szC; ++k) real[k] = ((double)(k % 17) - 8.0) / 3.0;
    const int p = f < l - 8 ? f : 2;
    oracle_encode(real, szC, p, l, plain);
    oracle_decode(plain, szC, p, l, dec);
    for (size_t k = 0; k < szC; ++k) CHECK(dec[k] <= real[k] && real[k] - dec[k] < 1.0 / (double)((u64)1 << p) * 1.0000001, "encode is floor");
    free(real); free(dec);
    free(x); free(y); free(back); free(X); free(Y); free(A); free(B); free(C); free(sa); free(sb); free(sc);
    free(Z); free(E); free(F); free(plain); free(Zr); free(a); free(bb); free(c); free(s); free(z);
    free(r); free(rt); free(rm); free(out);
}

int main(void)
{
    one_case(1, 1, 1, 1, 1, 64, 16, 1);
    one_case(2, 1, 5, 3, 7, 64, 16, 2);
    one_case(3, 2, 17, 9, 33, 64, 20, 3);
    one_case(5, 1, 8, 8, 8, 64, 1, 4);
    one_case(8, 1, 3, 2, 5, 64, 61, 5);
    one_case(3, 1, 6, 4, 5, 32, 12, 6);
    one_case(2, 3, 4, 4, 4, 16, 5, 7);
    one_case(3, 1, 4, 5, 6, 8, 3, 8);
    /* 128-bit ring: sharing and the plain product on exactly sized buffers */
    {
        enum { n = 3, M = 5, N = 4, K = 6 };
        u128 *P = (u128 *)malloc(sizeof(u128) * M * K), *Q = (u128 *)malloc(sizeof(u128) * K * N);
        u128 *R = (u128 *)malloc(sizeof(u128) * M * N), *sh = (u128 *)malloc(sizeof(u128) * n * M * K);
        u128 *back = (u128 *)malloc(sizeof(u128) * M * K);
        for (int k = 0; k < M * K; ++k) P[k] = ((u128)oracle_rand64(9, 1, 0, k) << 64) | oracle_rand64(9, 2, 0, k);
        for (int k = 0; k < K * N; ++k) Q[k] = ((u128)oracle_rand64(9, 3, 0, k) << 64) | oracle_rand64(9, 4, 0, k);
        oracle128_ring_matmul(P, Q, M, N, K, R);
        oracle128_share(P, M * K, n, 9, 1, sh);
        oracle128_open(sh, NULL, M * K, n, back);
        CHECK(memcmp(back, P, sizeof(u128) * M * K) == 0, "128-bit shares reconstruct");
        free(P); free(Q); free(R); free(sh); free(back);
    }
    if (failures) { printf("%d check(s) failed\n", failures); return 1; }
    printf("oracle sanitizer run ok\n");
    return 0;
}
