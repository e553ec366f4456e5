// Exact ring GEMM over Z_2^128 on the int8 matrix cores (the paper's second ring width: its own
// kernels multiply __int128, Section 6.1).
//
// Same decomposition as the 64-bit kernel with 16 balanced digits: a*b == sum_{i+j<=15} s_i t_j
// 256^(i+j) (mod 2^128), 136 digit pairs on v_mfma_i32_32x32x32_i8, 16 diagonal int32 accumulators,
// result sum_d (int128)D_d << 8d.  D_d needs 128-8d exact bits, so d <= 11 must not overflow:
// 12 * Ktot * 2^14 < 2^31  <=>  Ktot < 10923; for d >= 12 only the low 32 bits matter and wrapping
// leaves them right.  The host splits the inner dimension into chunks of at most 170 k-tiles per
// operand pair (Ktot <= 10880).
//
// Register budget decides the shape: 16 diagonals x 16 accumulator registers fill the 256 AGPRs with
// ONE 32x32 MFMA tile per wave, and the wave's 32 operand fragments (128 VGPRs) cannot be double
// buffered.  So: workgroup tile 64x64 (4 waves as 2x2), two LDS stages of 64 KB, loads of step s+1
// issued between the MFMAs of step s, fragments of a step read at its start.
#include "limb_common.hpp"

namespace spin {
namespace {

constexpr int kDigits128 = 16;
constexpr int kMaxChunkTiles128 = 170;    // 2*170*32 = 10880 < 10923 digit products per exact accumulator

struct Gemm128Args {
    const char *packA;   // [n+1][batch][nblkA][KT][16][1024]: slot 0 = E, slot 1+i = A_i
    const char *packB;   // [n+1][batch][nblkB][KT][16][1024]: slot 0 = F, slot 1+i = B_i'
    const u128 *C;       // [n][batch][M][N]  (or Z itself for the later k-chunks)
    u128 *Z;
    int n, batch, M, N;
    int nblkA, nblkB, KT;
    int kt0, ktn;        // this launch covers k-tiles [kt0, kt0+ktn) of both operand pairs
    int tilesM, tilesN;
};

struct Shape128 {
    static constexpr int ND = kDigits128;
    static constexpr int NSTAGE = 2;
    static constexpr int BM = 64, BN = 64;                       // 4 waves as 2 x 2, one 32x32 tile each
    static constexpr int FA = BM / 32 * ND, FB = BN / 32 * ND;   // fragments per stage: 32 + 32
    static constexpr int stage_bytes = (FA + FB) * kFrag;        // 64 KB
    static constexpr int lds_bytes = NSTAGE * stage_bytes;
    static constexpr int loads_per_wave = (FA + FB) / 4;         // 16
};

__global__ __launch_bounds__(256) void limb128_gemm_kernel(Gemm128Args g)
{
    using S = Shape128;
    constexpr int ND = S::ND;
    extern __shared__ __attribute__((aligned(1024))) char lds[];

    const int lane = threadIdx.x % 64;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    const int wm = wave / 2, wn = wave % 2;
    const TileId tile = map_tile(blockIdx.x, g.tilesM, g.tilesN, (long)g.tilesM * g.tilesN * g.n * g.batch);
    const int pb = tile.pb, tm = tile.tm, tn = tile.tn;
    const int party = pb / g.batch, b = pb % g.batch;

    // fragment streams: step < ktn uses (E, B_i'), step >= ktn uses (A_i, F)
    const size_t blk_stride = (size_t)g.KT * (ND * kFrag);
    const size_t slotA = (size_t)g.batch * g.nblkA * blk_stride;
    const size_t slotB = (size_t)g.batch * g.nblkB * blk_stride;
    const char *a_first = g.packA + (size_t)b * g.nblkA * blk_stride;      // E
    const char *a_second = a_first + (size_t)(1 + party) * slotA;          // A_i
    const char *b_second = g.packB + (size_t)b * g.nblkB * blk_stride;     // F
    const char *b_first = b_second + (size_t)(1 + party) * slotB;          // B_i'

    const int steps = 2 * g.ktn;
    const u32 lds0 = (u32)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
    const u32 lane16 = lane * 16;

    // Load cursor (scalar unit): this wave loads fragments f = 4q + wave, q < 16: block f / 16 = q / 4
    // of the tile and digit f % 16 = 4 (q % 4) + wave.
    const size_t kt0_off = (size_t)g.kt0 * (ND * kFrag) + wave * kFrag;
    const char *ld_a = a_first + (size_t)tm * (S::BM / 32) * blk_stride + kt0_off;
    const char *ld_b = b_first + (size_t)tn * (S::BN / 32) * blk_stride + kt0_off;
    const char *second_a = a_second + (size_t)tm * (S::BM / 32) * blk_stride + kt0_off;
    const char *second_b = b_second + (size_t)tn * (S::BN / 32) * blk_stride + kt0_off;
    int ld_left = g.ktn;
    const u32 ld_lds0 = lds0 + wave * kFrag;
    u32 ld_lds = ld_lds0;
    auto issue_load = [&](int q) {
        constexpr int qa = S::FA / 4, per_blk = ND / 4;
        const char *p = q < qa ? ld_a + (size_t)(q / per_blk) * blk_stride + (q % per_blk) * (4 * kFrag)
                               : ld_b + (size_t)((q - qa) / per_blk) * blk_stride + ((q - qa) % per_blk) * (4 * kFrag);
        load_fragment_to_lds(p, ld_lds + q * (4 * kFrag), lane16);
    };
    auto advance_load_cursor = [&]() {
        ld_a += ND * kFrag;
        ld_b += ND * kFrag;
        if (--ld_left == 0) { ld_a = second_a; ld_b = second_b; }
        ld_lds = ld_lds == ld_lds0 ? ld_lds0 + S::stage_bytes : ld_lds0;     // two stages
    };

    v16i acc[ND];
#pragma unroll
    for (int d = 0; d < ND; ++d) acc[d] = (v16i)(0);

    const char *rd_a = lds + (wm * ND) * kFrag + lane16;
    const char *rd_b = lds + (S::FA + wn * ND) * kFrag + lane16;
    int rd_stage = 0;

    // prologue: loads of step 0
#pragma unroll
    for (int q = 0; q < S::loads_per_wave; ++q) issue_load(q);
    advance_load_cursor();

    for (int s = 0; s < steps; ++s) {
        wait_loads<0>();                                 // this wave's loads of step s have landed
        workgroup_barrier();                             // ... everyone's; and every wave is done reading step s-1
        const char *pa = rd_a + rd_stage * S::stage_bytes, *pb_ = rd_b + rd_stage * S::stage_bytes;
        rd_stage ^= 1;
        v4i fa[ND], fb[ND];
#pragma unroll
        for (int d = 0; d < ND; ++d) {
            fb[d] = *(const v4i *)(pb_ + d * kFrag);
            if (d < 2) fa[d] = *(const v4i *)(pa + d * kFrag);
        }
#pragma unroll
        for (int d = 2; d < ND; ++d) fa[d] = *(const v4i *)(pa + d * kFrag);
        __builtin_amdgcn_sched_barrier(0);
        const bool more = s + 1 < steps;
        int slot = 0;
#pragma unroll
        for (int da = 0; da < ND; ++da)
#pragma unroll
            for (int db = 0; db + da < ND; ++db) {
                acc[da + db] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[da], fb[db], acc[da + db], 0, 0, 0);
                // the loads of step s+1 go into the other stage (free since the barrier above), one after
                // every 8th MFMA
                if (slot % 8 == 4 && slot / 8 < S::loads_per_wave) {
                    if (more) issue_load(slot / 8);
                    __builtin_amdgcn_sched_barrier(0);
                }
                ++slot;
            }
        if (more) advance_load_cursor();
    }

    // Recombine the diagonals and add C_i.  All C values are loaded before the first store, so that the
    // loads do not each wait out the store before them (C and Z may be the same buffer); tiles wholly
    // inside the matrix take a branch-free copy, in which the stores do not wait for each other either.
    const size_t mat = (size_t)g.M * g.N;
    const u128 *Cm = g.C + (size_t)pb * mat;
    u128 *Zm = g.Z + (size_t)pb * mat;
    const int col = tn * S::BN + wn * 32 + lane % 32;
    const int row0 = tm * S::BM + wm * 32 + 4 * (lane / 32);
    auto epilogue = [&](auto interior_c) {
        constexpr bool INTERIOR = decltype(interior_c)::value;
        u128 cv[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = row0 + 8 * (r / 4) + r % 4;
            cv[r] = (INTERIOR || (row < g.M && col < g.N)) ? Cm[(size_t)row * g.N + col] : (u128)0;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = row0 + 8 * (r / 4) + r % 4;
            u128 v = cv[r];
#pragma unroll
            for (int d = 0; d < ND; ++d) v += (u128)(__int128)acc[d][r] << (8 * d);
            if (INTERIOR || (row < g.M && col < g.N)) Zm[(size_t)row * g.N + col] = v;
        }
    };
    if ((tm + 1) * S::BM <= g.M && (tn + 1) * S::BN <= g.N) epilogue(std::true_type());
    else epilogue(std::false_type());
}

struct Plan128 {
    int KT, nblkA, nblkB, tilesM, tilesN;
    size_t packA_bytes, packB_bytes;
};
inline Plan128 make_plan128(int n, int batch, int M, int N, int K)
{
    Plan128 p;
    p.KT = ceil_div(K, 32);
    p.tilesM = ceil_div(M, Shape128::BM);
    p.tilesN = ceil_div(N, Shape128::BN);
    p.nblkA = p.tilesM * (Shape128::BM / 32);
    p.nblkB = p.tilesN * (Shape128::BN / 32);
    p.packA_bytes = (size_t)(n + 1) * batch * p.nblkA * p.KT * (kDigits128 * kFrag);
    p.packB_bytes = (size_t)(n + 1) * batch * p.nblkB * p.KT * (kDigits128 * kFrag);
    return p;
}

}  // namespace

size_t limb128_workspace_bytes(int n, int batch, int M, int N, int K)
{
    Plan128 p = make_plan128(n, batch, M, N, K);
    return p.packA_bytes + p.packB_bytes;
}

spin_status launch_matmul_limb128(const MatmulArgs128 &a, hipStream_t s)
{
    const Plan128 p = make_plan128(a.n, a.batch, a.M, a.N, a.K);
    char *packA = (char *)a.workspace;
    char *packB = packA + p.packA_bytes;
    launch_pack<u128>(a, packA, packB, p.nblkA, p.nblkB, p.KT, s);
    spin_status st = check_launch("spin128_beaver_matmul(pack)");
    if (st != SPIN_OK) return st;

    static OncePerDevice lds_allowed;
    st = allow_dynamic_lds((const void *)limb128_gemm_kernel, Shape128::lds_bytes, lds_allowed);
    if (st != SPIN_OK) return st;
    Gemm128Args g{packA, packB, a.C, a.Z, a.n, a.batch, a.M, a.N, p.nblkA, p.nblkB, p.KT, 0, 0, p.tilesM, p.tilesN};
    const long total = (long)p.tilesM * p.tilesN * a.n * a.batch;
    for (int kt0 = 0; kt0 < p.KT; kt0 += kMaxChunkTiles128) {
        g.kt0 = kt0;
        g.ktn = p.KT - kt0 < kMaxChunkTiles128 ? p.KT - kt0 : kMaxChunkTiles128;
        g.C = kt0 == 0 ? a.C : a.Z;                      // later chunks accumulate onto Z
        KernelTimer timer(SPIN_KERNEL_GEMM_LIMB, s);
        limb128_gemm_kernel<<<(unsigned)total, 256, Shape128::lds_bytes, s>>>(g);
        st = check_launch("spin128_beaver_matmul(limb gemm)");
        if (st != SPIN_OK) return st;
    }
    return SPIN_OK;
}

}  // namespace spin
