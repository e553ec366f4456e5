// Exact ring GEMM over Z_2^64 on the int8 matrix cores.
//
// Every uint64 a is rewritten as eight balanced digits s_0..s_7 in [-128,127]
// with  sum_i s_i 256^i == a  (mod 2^64)   [t = a + 0x80..80; s = t ^ 0x80..80].
// Then  a*b == sum_{i+j<=7} s_i t_j 256^(i+j)  (mod 2^64): the 28 digit pairs
// with i+j >= 8 are multiples of 2^64.  The 36 surviving pairs are int8 x int8
// products; pairs of one diagonal d = i+j share an int32 MFMA accumulator D_d,
// and the result is  sum_d (int64)D_d << 8d  (mod 2^64).
//
// int32 headroom: |s_i t_j| <= 2^14.  D_d needs 64-8d exact bits, so only
// d <= 3 must not overflow: (d+1) * Ktot * 2^14 < 2^31  <=>  Ktot < 2^15.
// For d >= 4 only the low 32 bits matter and the accumulators wrap (two's
// complement), which leaves those bits right.  The host splits the inner
// dimension into chunks of at most kMaxChunkTiles k-tiles per operand pair.
//
// Two kernels:
//  pack_left/right_kernel  open E (or F), convert E/A_i (or F/B_i') to digits and
//                store them as 1 KiB MFMA fragments: [slot][batch][blk][kt]
//                [digit][lane*16 + j] = digit of element (blk*32 + lane%32,
//                kt*32 + 16*(lane/32) + j).  Zero padded to whole tiles.
//  limb_gemm_kernel  per party: Z_i = C_i + [E | A_i] . [B_i' ; F], fragments
//                streamed global -> LDS with direct-to-LDS loads, 36 MFMAs per
//                32x32x32 step into 8 diagonal accumulators, recombined once.
#include "common.hpp"

// Interleave of one k-step of the GEMM (slots = MFMA index within the step, 72 per step for the 64x32
// wave tile): an LDS read after every RD_EVERY-th MFMA from slot 0, a direct-to-LDS load after every
// LD_EVERY-th MFMA from slot LD_FIRST.
#ifndef SPIN_TUNE_RD_EVERY
#define SPIN_TUNE_RD_EVERY 2
#endif
#ifndef SPIN_TUNE_LD_FIRST
#define SPIN_TUNE_LD_FIRST 13
#endif
#ifndef SPIN_TUNE_LD_EVERY
#define SPIN_TUNE_LD_EVERY 4
#endif

namespace spin {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int u32;

constexpr int kFrag = 1024;          // bytes of one 32x32 int8 fragment
constexpr int kDigits = 8;
constexpr int kMaxChunkTiles = 511;  // 2*511*32 = 32704 < 2^15 digit products per accumulator

// ------------------------------------------------------------------ pack ---
__device__ inline u64 to_digits(u64 a)
{
    return (a + 0x8080808080808080ull) ^ 0x8080808080808080ull;
}

// Transposes 16 digit-words (16 elements x 8 digits) into 8 rows of 16 bytes
// and stores row p at dst + p*kFrag.
__device__ inline void store_digit_rows(const u64 (&w)[16], char *dst)
{
#pragma unroll
    for (int half = 0; half < 2; ++half) {          // digits 0-3 from the low words, 4-7 from the high words
        u32 rows[4][4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            u32 w0 = (u32)(w[4 * q + 0] >> (32 * half)), w1 = (u32)(w[4 * q + 1] >> (32 * half));
            u32 w2 = (u32)(w[4 * q + 2] >> (32 * half)), w3 = (u32)(w[4 * q + 3] >> (32 * half));
            // 4x4 byte transpose with v_perm_b32 (selector 0-3: second operand, 4-7: first operand)
            u32 t0 = __builtin_amdgcn_perm(w1, w0, 0x05010400u);   // w0.b0 w1.b0 w0.b1 w1.b1
            u32 t1 = __builtin_amdgcn_perm(w1, w0, 0x07030602u);   // w0.b2 w1.b2 w0.b3 w1.b3
            u32 t2 = __builtin_amdgcn_perm(w3, w2, 0x05010400u);
            u32 t3 = __builtin_amdgcn_perm(w3, w2, 0x07030602u);
            rows[0][q] = __builtin_amdgcn_perm(t2, t0, 0x05040100u);
            rows[1][q] = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
            rows[2][q] = __builtin_amdgcn_perm(t3, t1, 0x05040100u);
            rows[3][q] = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
        }
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            v4i v = {(int)rows[p][0], (int)rows[p][1], (int)rows[p][2], (int)rows[p][3]};
            *(v4i *)(dst + (size_t)(half * 4 + p) * kFrag) = v;
        }
    }
}

struct PackArgs {
    const u64 *val;     // X or Y shares   [n][batch][R][Cc]
    const u64 *tri;     // A or B shares   [n][batch][R][Cc]
    char *pack;         // [n+1][batch][nblk][KT][8][1024]
    int n, batch;
    int rows, cols;     // source matrix is rows x cols, row-major
    int nblk, KT;       // blocks of 32 along the non-contracted axis; k-tiles of 32
};

// Both pack kernels make one pass over the 2n share streams of their side: every party's value and
// triple share is read exactly once; the opened matrix (E or F) accumulates in registers while each
// triple share is converted and stored as it arrives.  Slots: 0 = opened, 1 + i = party i's triple
// share (left side A_i; right side B_i, and for party 0 B_0 + F, which folds the public E.F term
// into party 0's first product).  One wave handles one 32 x 32 tile (blk, kt); blockIdx.z = batch.

// Right side: source K x N row-major, a fragment row is a matrix column, so the 16 consecutive k a
// lane needs are 16 strided loads whose lanes run along contiguous columns (256-byte segments).
template <int NP>
__global__ __launch_bounds__(256) void pack_right_kernel(PackArgs a)
{
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const long tile = (long)blockIdx.x * 4 + wave;
    if (tile >= (long)a.nblk * a.KT) return;
    const int blk = (int)(tile / a.KT), kt = (int)(tile % a.KT);
    const int b = blockIdx.z;
    const int K = a.rows, N = a.cols;
    const int col = blk * 32 + (lane % 32);
    const int k0 = kt * 32 + 16 * (lane / 32);
    const size_t mat = (size_t)K * N;
    const size_t party_stride = (size_t)a.batch * mat;
    auto frag = [&](int slot) -> char * {
        return a.pack + ((((size_t)slot * a.batch + b) * a.nblk + blk) * a.KT + kt) * (kDigits * kFrag) + lane * 16;
    };
    u64 opened[16], first[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) { opened[j] = 0; first[j] = 0; }
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        const u64 *v = a.val + (size_t)i * party_stride + (size_t)b * mat;
        const u64 *t = a.tri + (size_t)i * party_stride + (size_t)b * mat;
        u64 tv[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            tv[j] = 0;
            if (col < N && k0 + j < K) {
                const size_t e = (size_t)(k0 + j) * N + col;
                tv[j] = t[e];
                opened[j] += v[e] - tv[j];
            }
        }
        if (i == 0) {
#pragma unroll
            for (int j = 0; j < 16; ++j) first[j] = tv[j];
        } else {
#pragma unroll
            for (int j = 0; j < 16; ++j) tv[j] = to_digits(tv[j]);
            store_digit_rows(tv, frag(i + 1));
        }
    }
    u64 w[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) w[j] = to_digits(opened[j]);
    store_digit_rows(w, frag(0));
#pragma unroll
    for (int j = 0; j < 16; ++j) w[j] = to_digits(first[j] + opened[j]);
    store_digit_rows(w, frag(1));
}

// Left side: source M x K row-major, a fragment row is a matrix row.  Reading 16 consecutive k per
// lane directly would make every wave-wide load touch 64 different rows; instead a wave reads its
// tile as 4 rows x 256 contiguous bytes per load, sums the parties' shares in that layout, and turns
// each 32 x 32 tile through LDS (rows padded to 272 bytes, conflict-free for 16-byte accesses both
// ways) so that each lane ends up with the 16 consecutive k of one row that a fragment chunk needs.
template <int NP, bool VEC>
__global__ __launch_bounds__(256) void pack_left_kernel(PackArgs a)
{
    constexpr int kRowBytes = 272;
    __shared__ __attribute__((aligned(16))) char turn[4][32 * kRowBytes];
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    long tile = (long)blockIdx.x * 4 + wave;                // (blk, kt) pair
    const bool active = tile < (long)a.nblk * a.KT;
    if (!active) tile = 0;
    const int blk = (int)(tile / a.KT), kt = (int)(tile % a.KT);
    const int b = blockIdx.z;
    const int M = a.rows, K = a.cols;
    const size_t mat = (size_t)M * K;
    const size_t party_stride = (size_t)a.batch * mat;
    const int kk = kt * 32 + 2 * (lane % 16);               // this lane's two k of every row it loads
    auto frag = [&](int slot) -> char * {
        return a.pack + ((((size_t)slot * a.batch + b) * a.nblk + blk) * a.KT + kt) * (kDigits * kFrag) + lane * 16;
    };
    auto load2 = [&](const u64 *base, int row) -> u64x2 {  // elements (row, kk) and (row, kk+1), zero outside
        u64x2 v = {0, 0};
        if (row < M) {
            const u64 *p = base + (size_t)row * K + kk;
            if (VEC) { if (kk < K) v = *(const u64x2 *)p; }
            else { if (kk < K) v.x = p[0]; if (kk + 1 < K) v.y = p[1]; }
        }
        return v;
    };
    // lane -> LDS: written as (row 4j + lane/16, k pair lane%16), read back as (row lane%32, k 16*(lane/32)..)
    char *mine = turn[wave];
    auto turn_and_store = [&](const u64x2 (&v)[8], char *dst) {
        __syncthreads();                                    // the previous round's reads are done
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            u64x2 d = {to_digits(v[j].x), to_digits(v[j].y)};
            *(u64x2 *)(mine + (4 * j + lane / 16) * kRowBytes + (lane % 16) * 16) = d;
        }
        __syncthreads();
        u64 w[16];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            u64x2 d = *(const u64x2 *)(mine + (lane % 32) * kRowBytes + (lane / 32) * 128 + j * 16);
            w[2 * j] = d.x; w[2 * j + 1] = d.y;
        }
        if (active) store_digit_rows(w, dst);
    };

    u64x2 opened[8], first[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { opened[j] = (u64x2)(0); first[j] = (u64x2)(0); }
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        const u64 *v = a.val + (size_t)i * party_stride + (size_t)b * mat;
        const u64 *t = a.tri + (size_t)i * party_stride + (size_t)b * mat;
        u64x2 tv[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int row = blk * 32 + 4 * j + lane / 16;
            tv[j] = load2(t, row);
            opened[j] += load2(v, row) - tv[j];
        }
        if (i == 0) {
#pragma unroll
            for (int j = 0; j < 8; ++j) first[j] = tv[j];
        } else {
            turn_and_store(tv, frag(i + 1));
        }
    }
    turn_and_store(opened, frag(0));
    turn_and_store(first, frag(1));
}

// ------------------------------------------------------------------ GEMM ---
struct GemmArgs {
    const char *packA;   // [n+1][batch][nblkA][KT][8][1024]: slot 0 = E, slot 1+i = A_i
    const char *packB;   // [n+1][batch][nblkB][KT][8][1024]: slot 0 = F, slot 1+i = B_i'
    const u64 *C;        // [n][batch][M][N]  (or Z itself for the later k-chunks)
    u64 *Z;
    int n, batch, M, N;
    int nblkA, nblkB, KT;
    int kt0, ktn;        // this launch covers k-tiles [kt0, kt0+ktn) of both operand pairs
    int tilesM, tilesN;
};

template <int WM, int WN>
struct GemmShape {
    static constexpr int NSTAGE = 3;                             // LDS ring: one stage read, two in flight
    static constexpr int BM = 2 * 32 * WM, BN = 2 * 32 * WN;     // 4 waves as 2 x 2
    static constexpr int FA = BM / 32 * kDigits, FB = BN / 32 * kDigits;
    static constexpr int stage_bytes = (FA + FB) * kFrag;
    static constexpr int lds_bytes = NSTAGE * stage_bytes;
    static constexpr int loads_per_wave = (FA + FB) / 4;
    static constexpr int frags_per_wave = (WM + WN) * kDigits;   // LDS -> register reads per step
    static constexpr int mfma_per_step = 36 * WM * WN;
};

// One direct-to-LDS load: 64 lanes x 16 bytes from src + lane*16 to the LDS address lds_dst + lane*16.
// Issued through inline assembly so that the compiler's LDS-DMA bookkeeping does not serialise the
// software pipeline; completion is awaited explicitly (wait_loads) before the workgroup barrier.
__device__ inline void load_fragment_to_lds(const char *src, u32 lds_dst, u32 lane16)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(lane16), "s"(src), "s"(lds_dst) : "memory");
}
template <int N> __device__ inline void wait_loads() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }
__device__ inline void wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ inline void workgroup_barrier() { asm volatile("s_barrier" ::: "memory"); }

// Pipeline (per wave; step s covers one 32-deep k-tile of one operand pair):
//   G(s)  12 direct-to-LDS loads of this wave's share of step s into LDS stage s % 3
//   R(s)  24 ds_read_b128 of the wave's fragments of step s into registers
//   M(s)  72 MFMAs of step s
// Iteration s: [wait G(s+1); barrier]  then M(s) interleaved with R(s+1) and G(s+3).
// The barrier at the top of iteration s also tells every wave that all R(s) are done, so stage s % 3
// can be refilled by G(s+3).  Two groups of loads are in flight while a step computes.
template <int WM, int WN>
__global__ __launch_bounds__(256) void limb_gemm_kernel(GemmArgs g)
{
    using S = GemmShape<WM, WN>;
    extern __shared__ __attribute__((aligned(1024))) char lds[];

    const int lane = threadIdx.x % 64;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    const int wm = wave / 2, wn = wave % 2;

    // Workgroup ids are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of tiles so
    // that workgroups sharing an L2 also share operand fragments, and walk that range in 4-tile-tall
    // column strips.
    const int per_mat = g.tilesM * g.tilesN;
    const long total = (long)per_mat * g.n * g.batch;
    long id = blockIdx.x;
    {
        const long chunk = (total + 7) / 8;
        const long full = total - (chunk - 1) * 8;       // XCDs that own `chunk` tiles (the rest own chunk-1)
        const int xcd = (int)(id % 8);
        const long within = id / 8;
        id = xcd < full ? xcd * chunk + within : full * chunk + (xcd - full) * (chunk - 1) + within;
    }
    const int pb = (int)(id / per_mat);                  // party * batch + b
    int t = (int)(id % per_mat);
    const int party = pb / g.batch, b = pb % g.batch;
    constexpr int GROUP = 4;
    const int strip = t / (GROUP * g.tilesN);
    const int strip_h = min(GROUP, g.tilesM - strip * GROUP);
    t -= strip * GROUP * g.tilesN;
    const int tm = strip * GROUP + t % strip_h, tn = t / strip_h;

    // fragment streams: step < ktn uses (E, B_i'), step >= ktn uses (A_i, F)
    const size_t slotA = (size_t)g.batch * g.nblkA * g.KT * (kDigits * kFrag);
    const size_t slotB = (size_t)g.batch * g.nblkB * g.KT * (kDigits * kFrag);
    const char *a_first = g.packA + (size_t)b * g.nblkA * g.KT * (kDigits * kFrag);   // E
    const char *a_second = a_first + (size_t)(1 + party) * slotA;                      // A_i
    const char *b_second = g.packB + (size_t)b * g.nblkB * g.KT * (kDigits * kFrag);  // F
    const char *b_first = b_second + (size_t)(1 + party) * slotB;                      // B_i'

    const int steps = 2 * g.ktn;
    const u32 lds0 = (u32)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
    const u32 lane16 = lane * 16;

    // Load cursor: where the loads of the next step to be fetched come from and go to.  It lives on
    // the scalar unit and advances by one k-tile per step (no division, no per-load selects); at the
    // switch from the first operand pair to the second it jumps to the other fragment streams.
    // This wave loads fragments f = 4q + wave, q < loads_per_wave: row/column block f / 8 = q / 2 of
    // the tile and digit f % 8 = 4 (q % 2) + wave, so only q-dependent constants remain per load.
    const size_t blk_stride = (size_t)g.KT * (kDigits * kFrag);
    const size_t kt0_off = (size_t)g.kt0 * (kDigits * kFrag) + wave * kFrag;
    const char *ld_a = a_first + (size_t)tm * (S::BM / 32) * blk_stride + kt0_off;
    const char *ld_b = b_first + (size_t)tn * (S::BN / 32) * blk_stride + kt0_off;
    const char *second_a = a_second + (size_t)tm * (S::BM / 32) * blk_stride + kt0_off;
    const char *second_b = b_second + (size_t)tn * (S::BN / 32) * blk_stride + kt0_off;
    int ld_left = g.ktn;                                 // steps until the cursor switches operand pair
    u32 ld_lds = lds0 + wave * kFrag;                    // LDS destination of the cursor's stage
    const u32 lds_wrap = lds0 + wave * kFrag + (S::NSTAGE - 1) * S::stage_bytes;
    auto issue_load = [&](int q) {                       // q is a compile-time constant after unrolling
        constexpr int qa = S::FA / 4;                    // loads of left-operand fragments per wave
        const char *p = q < qa ? ld_a + (size_t)(q / 2) * blk_stride + (q % 2) * (4 * kFrag)
                               : ld_b + (size_t)((q - qa) / 2) * blk_stride + ((q - qa) % 2) * (4 * kFrag);
        load_fragment_to_lds(p, ld_lds + q * (4 * kFrag), lane16);
    };
    auto advance_load_cursor = [&]() {
        ld_a += kDigits * kFrag;
        ld_b += kDigits * kFrag;
        if (--ld_left == 0) { ld_a = second_a; ld_b = second_b; }
        ld_lds = ld_lds == lds_wrap ? lds_wrap - (S::NSTAGE - 1) * S::stage_bytes : ld_lds + S::stage_bytes;
    };

    v16i acc[WM][WN][kDigits];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int d = 0; d < kDigits; ++d) acc[i][j][d] = (v16i)(0);

    // fragment registers, double buffered: [buffer][B fragments then A fragments]; the read cursor
    // (two LDS pointers of this wave within the stage to be read next) cycles through the stages
    v4i fr[2][S::frags_per_wave];
    const char *rd_a = lds + (wm * WM * kDigits) * kFrag + lane16;
    const char *rd_b = lds + (S::FA + wn * WN * kDigits) * kFrag + lane16;
    const char *rd_wrap = rd_a + (S::NSTAGE - 1) * S::stage_bytes;
    auto read_fragment = [&](int q) -> v4i {             // q < WN*8: B fragment q; else A fragment q - WN*8
        return *(const v4i *)(q < WN * kDigits ? rd_b + q * kFrag : rd_a + (q - WN * kDigits) * kFrag);
    };
    auto advance_read_cursor = [&]() {
        const bool wrap = rd_a == rd_wrap;
        rd_a = wrap ? rd_a - (S::NSTAGE - 1) * S::stage_bytes : rd_a + S::stage_bytes;
        rd_b = wrap ? rd_b - (S::NSTAGE - 1) * S::stage_bytes : rd_b + S::stage_bytes;
    };

    // prologue: G(0), G(1), G(2); R(0)
#pragma unroll
    for (int q = 0; q < S::loads_per_wave; ++q) issue_load(q);
    advance_load_cursor();
#pragma unroll
    for (int q = 0; q < S::loads_per_wave; ++q) issue_load(q);
    advance_load_cursor();
    if (steps > 2) {
#pragma unroll
        for (int q = 0; q < S::loads_per_wave; ++q) issue_load(q);
        advance_load_cursor();
        wait_loads<2 * S::loads_per_wave>();
    } else {
        wait_loads<S::loads_per_wave>();
    }
    workgroup_barrier();
#pragma unroll
    for (int q = 0; q < S::frags_per_wave; ++q) fr[0][q] = read_fragment(q);
    advance_read_cursor();

    // One step.  CUR: register buffer holding this step.  LOAD: the step three ahead exists.
    // NEXT: the next step exists.  MORE: the step two ahead exists (its loads stay in flight across the wait).
    auto iteration = [&](auto cur_c, auto load_c, auto next_c, auto more_c) {
        constexpr int cur = decltype(cur_c)::value, nxt = cur ^ 1;
        constexpr bool LOAD = decltype(load_c)::value, NEXT = decltype(next_c)::value, MORE = decltype(more_c)::value;
        if (NEXT) {
            if (MORE) wait_loads<S::loads_per_wave>(); else wait_loads<0>();
        }
        wait_lds();
        workgroup_barrier();
        int slot = 0;
#pragma unroll
        for (int da = 0; da < kDigits; ++da)
#pragma unroll
            for (int db = 0; db + da < kDigits; ++db)
#pragma unroll
                for (int i = 0; i < WM; ++i)
#pragma unroll
                    for (int j = 0; j < WN; ++j) {
                        acc[i][j][da + db] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                            fr[cur][WN * kDigits + i * kDigits + da], fr[cur][j * kDigits + db], acc[i][j][da + db],
                            0, 0, 0);
                        // Between the MFMAs: the next step's LDS reads (every rd_every-th slot from the
                        // start, so they are done long before the next barrier), the global loads of the
                        // step three ahead (every ld_every-th slot from ld_first), and the two cursor
                        // updates, so that the last MFMAs of a step and the barrier that follows have no
                        // scalar work between them.  sched_barrier pins this order: left alone, the
                        // scheduler sinks each read next to its first use and the MFMA pipe then waits
                        // out the LDS latency.
                        constexpr int rd_every = SPIN_TUNE_RD_EVERY;
                        constexpr int rd_last = rd_every * (S::frags_per_wave - 1);
                        constexpr int ld_first = SPIN_TUNE_LD_FIRST;
                        constexpr int ld_every = SPIN_TUNE_LD_EVERY;
                        constexpr int ld_last = ld_first + ld_every * (S::loads_per_wave - 1);
                        static_assert(rd_every >= 1 && ld_every >= 1 && ld_last + 1 < S::mfma_per_step &&
                                      rd_last + 1 < S::mfma_per_step, "tile too small for this interleave");
                        if (NEXT && slot % rd_every == 0 && slot <= rd_last) {
                            fr[nxt][slot / rd_every] = read_fragment(slot / rd_every);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        if (NEXT && slot == rd_last + 1) {
                            advance_read_cursor();
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        if (LOAD && slot >= ld_first && (slot - ld_first) % ld_every == 0 && slot <= ld_last) {
                            issue_load((slot - ld_first) / ld_every);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        if (LOAD && slot == ld_last + 1) {
                            advance_load_cursor();
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        ++slot;
                    }
    };
    using T = std::true_type;
    using F = std::false_type;
    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;
    int s = 0;
    for (; s + 4 < steps; s += 2) {                       // steps is even; both halves have all neighbours
        iteration(B0(), T(), T(), T());
        iteration(B1(), T(), T(), T());
    }
    if (steps >= 4) {
        iteration(B0(), T(), T(), T());                   // step steps-4: loads the last step
        iteration(B1(), F(), T(), T());
    }
    iteration(B0(), F(), T(), F());                       // step steps-2
    iteration(B1(), F(), F(), F());                       // step steps-1

    // recombine the diagonals and add C_i
    const size_t mat = (size_t)g.M * g.N;
    const u64 *Cm = g.C + (size_t)pb * mat;
    u64 *Zm = g.Z + (size_t)pb * mat;
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int col = tn * S::BN + (wn * WN + j) * 32 + lane % 32;
            const int row0 = tm * S::BM + (wm * WM + i) * 32 + 4 * (lane / 32);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = row0 + 8 * (r / 4) + r % 4;
                u64 v = 0;
#pragma unroll
                for (int d = 0; d < kDigits; ++d) v += (u64)(int64_t)acc[i][j][d][r] << (8 * d);
                if (row < g.M && col < g.N) Zm[(size_t)row * g.N + col] = Cm[(size_t)row * g.N + col] + v;
            }
        }
}

// ------------------------------------------------------------------ host ---
constexpr int kWM = 2, kWN = 1;
using Shape = GemmShape<kWM, kWN>;

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

struct Plan {
    int KT, nblkA, nblkB, tilesM, tilesN;
    size_t packA_bytes, packB_bytes;
};
inline Plan make_plan(int n, int batch, int M, int N, int K)
{
    Plan p;
    p.KT = ceil_div(K, 32);
    p.tilesM = ceil_div(M, Shape::BM);
    p.tilesN = ceil_div(N, Shape::BN);
    p.nblkA = p.tilesM * (Shape::BM / 32);
    p.nblkB = p.tilesN * (Shape::BN / 32);
    p.packA_bytes = (size_t)(n + 1) * batch * p.nblkA * p.KT * (kDigits * kFrag);
    p.packB_bytes = (size_t)(n + 1) * batch * p.nblkB * p.KT * (kDigits * kFrag);
    return p;
}

}  // namespace

size_t limb_workspace_bytes(int n, int batch, int M, int N, int K)
{
    Plan p = make_plan(n, batch, M, N, K);
    return p.packA_bytes + p.packB_bytes;
}

spin_status launch_matmul_limb(const MatmulArgs &a, hipStream_t s)
{
    const Plan p = make_plan(a.n, a.batch, a.M, a.N, a.K);
    char *packA = (char *)a.workspace;
    char *packB = packA + p.packA_bytes;

    PackArgs pa{a.X, a.A, packA, a.n, a.batch, a.M, a.K, p.nblkA, p.KT};
    PackArgs pb{a.Y, a.B, packB, a.n, a.batch, a.K, a.N, p.nblkB, p.KT};
    for_party_count(a.n, [&](auto np) {
        constexpr int NP = decltype(np)::value;
        KernelTimer timer(SPIN_KERNEL_PACK, s);
        dim3 ga((unsigned)(((long)p.nblkA * p.KT + 3) / 4), 1, a.batch);
        if (a.K % 2 == 0) pack_left_kernel<NP, true><<<ga, 256, 0, s>>>(pa);   // rows 16-byte aligned
        else pack_left_kernel<NP, false><<<ga, 256, 0, s>>>(pa);
        dim3 gb((unsigned)(((long)p.nblkB * p.KT + 3) / 4), 1, a.batch);
        pack_right_kernel<NP><<<gb, 256, 0, s>>>(pb);
    });
    spin_status st = check_launch("spin_beaver_matmul(pack)");
    if (st != SPIN_OK) return st;

    static bool attr_set = false;
    auto kernel = limb_gemm_kernel<kWM, kWN>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           Shape::lds_bytes);
        if (e != hipSuccess) { note_hip_error(e, "hipFuncSetAttribute"); return SPIN_EHIP; }
        attr_set = true;
    }
    GemmArgs g{packA, packB, a.C, a.Z, a.n, a.batch, a.M, a.N, p.nblkA, p.nblkB, p.KT, 0, 0, p.tilesM, p.tilesN};
    const long total = (long)p.tilesM * p.tilesN * a.n * a.batch;
    for (int kt0 = 0; kt0 < p.KT; kt0 += kMaxChunkTiles) {
        g.kt0 = kt0;
        g.ktn = p.KT - kt0 < kMaxChunkTiles ? p.KT - kt0 : kMaxChunkTiles;
        g.C = kt0 == 0 ? a.C : a.Z;                      // later chunks accumulate onto Z
        KernelTimer timer(SPIN_KERNEL_GEMM_LIMB, s);
        kernel<<<(unsigned)total, 256, Shape::lds_bytes, s>>>(g);
    }
    return check_launch("spin_beaver_matmul(limb gemm)");
}

}  // namespace spin
