// Measurement aid: what int8 MFMA rate does the chip sustain on given operand data?
//
// A register-only loop of the limb GEMM's instruction pattern: per iteration every wave issues the 72
// v_mfma_i32_32x32x32_i8 of one k-step of the 64-bit kernel (two 32x32 tiles, 36 digit pairs, eight
// diagonal accumulators each) on 24 operand fragments it loaded once, with no LDS or memory traffic
// inside the loop.  On MI355X the result depends strongly on the operand bytes: all-zero operands run
// close to the nominal 5.0 POP/s, uniformly random bytes (what the digits of masked shares are) far
// below it, because the chip lowers its clock under that load.  The benchmark reports both figures next
// to the GEMM kernel's own rate.
#include "limb_common.hpp"

namespace spin {
namespace {

__global__ __launch_bounds__(256) void mfma_probe_kernel(const v4i *__restrict__ operands, int iters,
                                                        u64 *__restrict__ sink)
{
    const int lane = threadIdx.x % 64;
    v4i fa[2][8], fb[8];                                 // 16 left fragments (two tiles), 8 right fragments
#pragma unroll
    for (int d = 0; d < 8; ++d) {
        fa[0][d] = operands[d * 64 + lane];
        fa[1][d] = operands[(8 + d) * 64 + lane];
        fb[d] = operands[(16 + d) * 64 + lane];
    }
    v16i acc[2][8];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int d = 0; d < 8; ++d) acc[t][d] = (v16i)(0);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int da = 0; da < 8; ++da)
#pragma unroll
            for (int db = 0; db + da < 8; ++db)
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    acc[t][da + db] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[t][da], fb[db], acc[t][da + db], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
    }
    int sum = 0;                                         // wraps like the accumulators
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int d = 0; d < 8; ++d)
#pragma unroll
            for (int r = 0; r < 16; ++r) sum += acc[t][d][r];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = (u64)(int64_t)sum;
}

}  // namespace

spin_status launch_mfma_probe(const u64 *operands, int blocks, int iters, u64 *sink, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_PROBE, s);
    mfma_probe_kernel<<<blocks, 256, 0, s>>>((const v4i *)operands, iters, sink);
    return check_launch("spin_probe_mfma");
}

}  // namespace spin
