// Baseline ring GEMM on the vector ALU: Z_i = C_i + E.B_i' + A_i.F with native
// 64-bit (for Z_2^32 32-bit, for Z_2^128 __int128) multiply-add, LDS-tiled (Section 6.1's design point -- native int64
// arithmetic staged through shared memory -- kept as the reference path the
// limb-MFMA path is measured against).  B_0' = B_0 + F folds party 0's public
// E.F term into its first product.
#include "common.hpp"

namespace spin {
namespace {

constexpr int TM = 64, TN = 64, TK = 16;   // workgroup tile; 256 threads, 4x4 outputs each
constexpr int PADA = 2;

// YT: the right operands F and B_i are stored [N][K] (a transposed right operand, as K in Q.K^T).
template <class T, bool YT>
__global__ __launch_bounds__(256) void valu_gemm_kernel(int n, int batch, int M, int N, int K,
                                                       const T *__restrict__ E, const T *__restrict__ F,
                                                       const T *__restrict__ A, const T *__restrict__ B,
                                                       const T *C, T *Z)
{
    __shared__ T As[TK][TM + PADA];   // k-major so that a thread's 4 rows are contiguous
    __shared__ T Bs[TK][TN];

    const int pb = blockIdx.z;          // party * batch + b
    const int party = pb / batch, b = pb % batch;
    const int tiles_n = (N + TN - 1) / TN;           // blockIdx.x = tile row * tiles_n + tile column
    const int m0 = (int)(blockIdx.x / tiles_n) * TM, n0 = (int)(blockIdx.x % tiles_n) * TN;
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;

    const T *Eb = E + (size_t)b * M * K;
    const T *Fb = F + (size_t)b * K * N;
    const T *Ai = A + (size_t)pb * M * K;
    const T *Bi = B + (size_t)pb * K * N;

    T acc[4][4] = {};
    const int ksteps = (K + TK - 1) / TK;
    for (int step = 0; step < 2 * ksteps; ++step) {
        const bool second = step >= ksteps;          // first E.B_i', then A_i.F
        const int k0 = (second ? step - ksteps : step) * TK;
        const T *left = second ? Ai : Eb;
        const T *right = second ? Fb : Bi;
        {   // left tile: 64 rows x 16 k, 4 elements per thread, stored transposed
            int row = threadIdx.x / 4, kk = (threadIdx.x % 4) * 4;
#pragma unroll
            for (int j = 0; j < 4; ++j) {                // unconditional loads: out of range reads element 0, then zero
                int gm = m0 + row, gk = k0 + kk + j;
                const bool ok = gm < M && gk < K;
                const T v = left[ok ? (size_t)gm * K + gk : 0];
                As[kk + j][row] = ok ? v : (T)0;
            }
        }
        {   // right tile: 16 k x 64 cols
            int kk = threadIdx.x / 16, col = (threadIdx.x % 16) * 4;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int gk = k0 + kk, gn = n0 + col + j;
                const bool ok = gk < K && gn < N;
                const size_t e = !ok ? 0 : YT ? (size_t)gn * K + gk : (size_t)gk * N + gn;
                T v = right[e];
                if (!second && party == 0) v += Fb[e];
                Bs[kk][col + j] = ok ? v : (T)0;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < TK; ++kk) {
            T av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bv[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += av[i] * bv[j];
        }
        __syncthreads();
    }
    // all C values are loaded before the first store (C and Z may be the same buffer, so interleaved
    // loads would each wait out the store before them)
    const T *Ci = C + (size_t)pb * M * N;
    T *Zi = Z + (size_t)pb * M * N;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int gm = m0 + ty * 4 + i, gn = n0 + tx * 4 + j;
            if (gm < M && gn < N) acc[i][j] += Ci[(size_t)gm * N + gn];
        }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int gm = m0 + ty * 4 + i, gn = n0 + tx * 4 + j;
            if (gm < M && gn < N) Zi[(size_t)gm * N + gn] = acc[i][j];
        }
}

}  // namespace

size_t valu_workspace_bytes(int, int batch, int M, int N, int K, int elem_bytes)
{
    return (size_t)elem_bytes * batch * ((size_t)M * K + (size_t)K * N);
}

template <class T> spin_status launch_matmul_valu(const MatmulArgsT<T> &a, hipStream_t s)
{
    T *E = (T *)a.workspace;
    T *F = E + (size_t)a.batch * a.M * a.K;
    spin_status st = launch_open<T>(a.X, a.A, (size_t)a.batch * a.M * a.K, a.n, E, s);
    if (st != SPIN_OK) return st;
    st = launch_open<T>(a.Y, a.B, (size_t)a.batch * a.K * a.N, a.n, F, s);
    if (st != SPIN_OK) return st;
    KernelTimer timer(SPIN_KERNEL_GEMM_VALU, s);
    // tiles on the x axis (the y axis holds at most 65535 blocks, fewer than the tile rows of a long operand)
    dim3 grid((unsigned)((size_t)((a.N + TN - 1) / TN) * ((a.M + TM - 1) / TM)), 1, a.n * a.batch);
    if (a.y_transposed) valu_gemm_kernel<T, true><<<grid, 256, 0, s>>>(a.n, a.batch, a.M, a.N, a.K, E, F, a.A, a.B, a.C, a.Z);
    else valu_gemm_kernel<T, false><<<grid, 256, 0, s>>>(a.n, a.batch, a.M, a.N, a.K, E, F, a.A, a.B, a.C, a.Z);
    return check_launch("spin_beaver_matmul(valu)");
}
template spin_status launch_matmul_valu<u32>(const MatmulArgsT<u32> &, hipStream_t);
template spin_status launch_matmul_valu<u64>(const MatmulArgsT<u64> &, hipStream_t);
template spin_status launch_matmul_valu<u128>(const MatmulArgsT<u128> &, hipStream_t);

}  // namespace spin
