/*
 * The boundary used from plain C, with no Python and no torch in the process: device buffers from
 * hipMalloc, the five calls of include/spin.h on a small 3-party case (ragged sizes, both GEMM paths), and
 * the results compared word for word with the CPU oracle's C functions.  Built and run by
 * tests/test_gpu_c_abi.py; prints "c abi ok" and exits 0 on success.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "spin.h"

typedef uint64_t u64;

/* oracle/spin_oracle.c */
extern void oracle_share(const u64 *x, size_t count, int n, int l, u64 seed, u64 stream, u64 *shares);
extern void oracle_dealer_matmul(int n, int batch, int M, int N, int K, int l, u64 seed, u64 sA, u64 sB, u64 sC,
                                 u64 *A, u64 *B, u64 *C, u64 *scratchA, u64 *scratchB, u64 *scratchC);
extern void oracle_beaver_matmul(int n, int batch, int M, int N, int K, int l, const u64 *X, const u64 *Y,
                                 const u64 *A, const u64 *B, const u64 *C, u64 *Z, u64 *E_out, u64 *F_out,
                                 const int *rows, int nrows);
extern void oracle_trunc_dealer(int n, size_t count, int l, int f, u64 seed, u64 sR, u64 sT, u64 sM,
                                u64 *r_sh, u64 *rtop_sh, u64 *rmsb_sh, u64 *scratch);
extern void oracle_trunc(int n, size_t count, int l, int f, const u64 *x, const u64 *r, const u64 *r_top,
                         const u64 *r_msb, u64 *out);
extern void oracle_dealer_mul(int n, size_t count, int l, u64 seed, u64 sA, u64 sB, u64 sC, u64 *a, u64 *b, u64 *c,
                              u64 *scratch);
extern void oracle_beaver_mul(int n, size_t count, int l, const u64 *x, const u64 *y, const u64 *a, const u64 *b,
                              const u64 *c, u64 *z);
extern void oracle_open(const u64 *shares, const u64 *mask_sh, size_t count, int n, int l, u64 *out);

#define HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(2); } } while (0)
#define SPIN(x) do { spin_status s_ = (x); if (s_ != SPIN_OK) { printf("%s failed: %s %s\n", #x, spin_status_string(s_), spin_last_hip_error()); exit(3); } } while (0)

static u64 *host(size_t words) { u64 *p = (u64 *)calloc(words, 8); if (!p) exit(4); return p; }
static u64 *dev(size_t words) { void *p; HIP(hipMalloc(&p, words * 8)); return (u64 *)p; }
static u64 *to_dev(const u64 *h, size_t words) { u64 *d = dev(words); HIP(hipMemcpy(d, h, words * 8, hipMemcpyHostToDevice)); return d; }
static void expect(const char *what, const u64 *d, const u64 *want, size_t words)
{
    u64 *got = host(words);
    HIP(hipMemcpy(got, d, words * 8, hipMemcpyDeviceToHost));
    for (size_t k = 0; k < words; ++k)
        if (got[k] != want[k]) { printf("%s: word %zu is %016llx, oracle says %016llx\n", what, k, (unsigned long long)got[k], (unsigned long long)want[k]); exit(1); }
    free(got);
}

int main(void)
{
    const int n = 3, batch = 2, M = 70, N = 45, K = 33, f = 16, l = 64;
    const u64 seed = 0xC0FFEE;
    const size_t szA = (size_t)batch * M * K, szB = (size_t)batch * K * N, szC = (size_t)batch * M * N;
    hipStream_t stream;
    HIP(hipStreamCreate(&stream));

    /* plaintext ring elements: small signed values at 2f fractional bits stay inside the truncation range */
    u64 *x = host(szA), *y = host(szB);
    for (size_t k = 0; k < szA; ++k) x[k] = (u64)(int64_t)((int64_t)(k * 2654435761u % 200001) - 100000);
    for (size_t k = 0; k < szB; ++k) y[k] = (u64)(int64_t)((int64_t)(k * 40503u % 131071) - 65535);

    /* share on the GPU and in the oracle */
    u64 *X = host(n * szA), *Y = host(n * szB);
    oracle_share(x, szA, n, l, seed, 1, X);
    oracle_share(y, szB, n, l, seed, 2, Y);
    u64 *dx = to_dev(x, szA), *dy = to_dev(y, szB), *dX = dev(n * szA), *dY = dev(n * szB);
    SPIN(spin_share(dx, szA, n, seed, 1, dX, stream));
    SPIN(spin_share(dy, szB, n, seed, 2, dY, stream));
    HIP(hipStreamSynchronize(stream));
    expect("spin_share X", dX, X, n * szA);
    expect("spin_share Y", dY, Y, n * szB);

    /* triples from the oracle's dealer; Beaver matmul on both paths */
    u64 *A = host(n * szA), *B = host(n * szB), *C = host(n * szC);
    u64 *sa = host(szA), *sb = host(szB), *sc = host(szC);
    oracle_dealer_matmul(n, batch, M, N, K, l, seed, 3, 4, 5, A, B, C, sa, sb, sc);
    u64 *Z = host(n * szC), *E = host(szA), *F = host(szB);
    oracle_beaver_matmul(n, batch, M, N, K, l, X, Y, A, B, C, Z, E, F, NULL, 0);
    u64 *dA = to_dev(A, n * szA), *dB = to_dev(B, n * szB), *dC = to_dev(C, n * szC), *dZ = dev(n * szC);
    u64 *dE = dev(szA);
    SPIN(spin_open(dX, dA, szA, n, dE, stream));
    HIP(hipStreamSynchronize(stream));
    expect("spin_open (E = X - A)", dE, E, szA);
    for (int path = 0; path < 2; ++path) {
        size_t ws_bytes = spin_beaver_matmul_workspace_bytes(n, batch, M, N, K, (spin_gemm_path)path);
        void *ws;
        if (ws_bytes == 0) { printf("workspace query failed\n"); return 5; }
        HIP(hipMalloc(&ws, ws_bytes));
        HIP(hipMemsetAsync(dZ, 0xEE, n * szC * 8, stream));
        SPIN(spin_beaver_matmul(n, batch, M, N, K, dX, dY, dA, dB, dC, dZ, (spin_gemm_path)path, ws, ws_bytes, stream));
        HIP(hipStreamSynchronize(stream));
        expect(path == 0 ? "spin_beaver_matmul (limb)" : "spin_beaver_matmul (valu)", dZ, Z, n * szC);
        /* too small a workspace is refused before anything is launched */
        if (spin_beaver_matmul(n, batch, M, N, K, dX, dY, dA, dB, dC, dZ, (spin_gemm_path)path, ws, ws_bytes - 1, stream) != SPIN_EWORKSPACE) {
            printf("short workspace was not refused\n");
            return 6;
        }
        HIP(hipFree(ws));
    }

    /* truncation of the product, then an elementwise Beaver multiplication with Z itself */
    u64 *r = host(n * szC), *rt = host(n * szC), *rm = host(n * szC), *scr = host(szC), *T = host(n * szC);
    oracle_trunc_dealer(n, szC, l, f, seed, 6, 7, 8, r, rt, rm, scr);
    oracle_trunc(n, szC, l, f, Z, r, rt, rm, T);
    u64 *dr = to_dev(r, n * szC), *drt = to_dev(rt, n * szC), *drm = to_dev(rm, n * szC), *dT = dev(n * szC);
    SPIN(spin_trunc(n, szC, f, dZ, dr, drt, drm, dT, stream));
    HIP(hipStreamSynchronize(stream));
    expect("spin_trunc", dT, T, n * szC);

    u64 *a = host(n * szC), *b = host(n * szC), *c = host(n * szC), *W = host(n * szC);
    oracle_dealer_mul(n, szC, l, seed, 9, 10, 11, a, b, c, scr);
    oracle_beaver_mul(n, szC, l, T, Z, a, b, c, W);
    u64 *da = to_dev(a, n * szC), *db = to_dev(b, n * szC), *dc = to_dev(c, n * szC);
    SPIN(spin_beaver_mul(n, szC, dT, dZ, da, db, dc, dT, stream));       /* in place on its first operand */
    HIP(hipStreamSynchronize(stream));
    expect("spin_beaver_mul", dT, W, n * szC);

    /* reconstruction of the product through the library equals the oracle's */
    u64 *opened = host(szC), *dO = dev(szC);
    oracle_open(W, NULL, szC, n, l, opened);
    SPIN(spin_open(dT, NULL, szC, n, dO, stream));
    HIP(hipStreamSynchronize(stream));
    expect("spin_open", dO, opened, szC);

    printf("c abi ok\n");
    return 0;
}
