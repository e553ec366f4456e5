// Exact ring GEMM over Z_2^64 (and, with four digits, Z_2^32) on the int8 matrix cores.
//
// Z_2^64: every uint64 a is rewritten as eight balanced digits s_0..s_7 in [-128,127]
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
// dimension into chunks of at most 511 k-tiles per operand pair.
//
// Z_2^32 (the Fixed32 representation of Section 7.1): four digits, the 10 pairs with i+j <= 3, four
// diagonals; every diagonal needs at most 32 exact bits, so wrapping accumulators are always right
// and the inner dimension is never split.
//
// Kernels:
//  pack_left/right_kernel (limb_common.hpp)  open E (or F), convert E/A_i (or F/B_i') to
//                digits and store them as 1 KiB MFMA fragments.
//  limb_gemm_kernel  per party: Z_i = C_i + [E | A_i] . [B_i' ; F], fragments
//                streamed global -> LDS with direct-to-LDS loads, 36 MFMAs per
//                32x32x32 step into 8 diagonal accumulators, recombined once.
//  limb_gemm_rows_kernel  products with few column tiles (N <= 64; attention shapes), at most three
//                parties: no left pack at all -- a producer wave streams the raw X_j, A_j tiles into LDS
//                and opens E, one consumer wave per party converts its A_p in registers and runs the MFMAs.
//  *_grouped_kernel  the same bodies for several products of different shapes in one launch
//                (spin_beaver_matmul_grouped), the products found through a table in the kernel arguments.
#include <algorithm>
#include <vector>

#include "limb_common.hpp"

namespace spin {
namespace {

// Per ring: digits, workgroup shape (waves are 2 x 2, each WM x WN MFMA tiles of 32 x 32; ND * WM * WN
// * 16 accumulator registers <= 256), longest run of k-tiles one launch may accumulate, and the
// interleave of one k-step (slots = MFMA index within the step): an LDS read after every rd_every-th
// MFMA from slot 0, a direct-to-LDS load after every ld_every-th MFMA from slot ld_first.
template <class T> struct Ring;
template <> struct Ring<u64> {
    static constexpr int WM = 2, WN = 1;
    static constexpr int max_chunk_tiles = 511;        // 2*511*32 = 32704 < 2^15 digit products per accumulator
    static constexpr int rd_every = 2, ld_first = 13, ld_every = 4;   // 72 MFMAs, 24 reads, 12 loads per step
};
template <> struct Ring<u32> {
    static constexpr int WM = 2, WN = 2;
    static constexpr int max_chunk_tiles = 1 << 20;    // no headroom limit; keeps the step count an int
    static constexpr int rd_every = 2, ld_first = 5, ld_every = 4;   // 40 MFMAs, 16 reads, 8 loads per step
};

// ------------------------------------------------------------------ GEMM ---
template <class T> struct GemmArgs {
    const char *packA;   // [n+1][batch][nblkA][KT][ND][1024]: slot 0 = E, slot 1+i = A_i
    const char *packB;   // [n+1][batch][nblkB][KT][ND][1024]: slot 0 = F, slot 1+i = B_i'
    const T *C;          // [n][batch][M][N]  (or Z itself for the later k-chunks)
    T *Z;
    int n, batch, M, N;
    int nblkA, nblkB, KT;
    int kt0, ktn;        // this launch covers k-tiles [kt0, kt0+ktn) of both operand pairs
    int tilesM, tilesN;
    int splits;          // workgroups per output tile: each takes split_steps of the 2*ktn k-steps and, when
    int split_steps;     // splits > 1, adds its part onto Z atomically (Z then starts out as C)
};

template <class T>
struct GemmShape {
    static constexpr int ND = sizeof(T);                         // digits per ring element
    static constexpr int WM = Ring<T>::WM, WN = Ring<T>::WN;
    static constexpr int NSTAGE = 3;                             // LDS ring: one stage read, two in flight
    static constexpr int BM = 2 * 32 * WM, BN = 2 * 32 * WN;     // 4 waves as 2 x 2
    static constexpr int FA = BM / 32 * ND, FB = BN / 32 * ND;
    static constexpr int stage_bytes = (FA + FB) * kFrag;
    static constexpr int lds_bytes = NSTAGE * stage_bytes;
    static constexpr int loads_per_wave = (FA + FB) / 4;
    static constexpr int frags_per_wave = (WM + WN) * ND;        // LDS -> register reads per step
    static constexpr int mfma_per_step = ND * (ND + 1) / 2 * WM * WN;
    static_assert(ND * WM * WN * 16 <= 256, "accumulators exceed the AGPR file");
};

// sum_d D_d 256^d (mod 2^(8 ND)) of the diagonal sums D_d held as int32: the low four diagonals as signed
// 64-bit multiply-adds (256^d fits an int32), the high four only reach the upper word, where they are plain
// 32-bit shifts and adds.  About ten instructions per element where shifting every sign-extended term
// through 64 bits takes forty.
__device__ inline u64 recombine_diagonals(int d0, int d1, int d2, int d3, int d4, int d5, int d6, int d7)
{
    long long low = (long long)d0;
    low += (long long)d1 * (1 << 8);
    low += (long long)d2 * (1 << 16);
    low += (long long)d3 * (1 << 24);
    const u32 high = (u32)((u64)low >> 32) + (u32)d4 + ((u32)d5 << 8) + ((u32)d6 << 16) + ((u32)d7 << 24);
    return ((u64)high << 32) | (u32)low;
}
__device__ inline u32 recombine_diagonals(int d0, int d1, int d2, int d3)
{
    return (u32)d0 + ((u32)d1 << 8) + ((u32)d2 << 16) + ((u32)d3 << 24);
}

__device__ inline void ring_atomic_add(u64 *p, u64 v) { atomicAdd((unsigned long long *)p, (unsigned long long)v); }
__device__ inline void ring_atomic_add(u32 *p, u32 v) { atomicAdd((unsigned int *)p, (unsigned int)v); }

// Pipeline (per wave; step s covers one 32-deep k-tile of one operand pair; counts for Z_2^64):
//   G(s)  12 direct-to-LDS loads of this wave's share of step s into LDS stage s % 3
//   R(s)  24 ds_read_b128 of the wave's fragments of step s into registers
//   M(s)  72 MFMAs of step s
// Iteration s: [wait G(s+1); barrier]  then M(s) interleaved with R(s+1) and G(s+3).
// The barrier at the top of iteration s also tells every wave that all R(s) are done, so stage s % 3
// can be refilled by G(s+3).  Two groups of loads are in flight while a step computes.
template <class T>
__device__ __forceinline__ void limb_gemm_body(const GemmArgs<T> &g, unsigned block)
{
    using S = GemmShape<T>;
    constexpr int kDigits = S::ND, WM = S::WM, WN = S::WN;
    extern __shared__ __attribute__((aligned(1024))) char lds[];

    const int lane = threadIdx.x % 64;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    const int wm = wave / 2, wn = wave % 2;

    // work item = (split, tile), tiles fastest: neighbours on an XCD work on neighbouring tiles of one k-range
    const long tiles_total = (long)g.tilesM * g.tilesN * g.n * g.batch;
    const long item = xcd_contiguous_id(block, tiles_total * g.splits);
    const int split = (int)(item / tiles_total);
    const TileId tile = tile_of(item % tiles_total, g.tilesM, g.tilesN);
    const int pb = tile.pb, tm = tile.tm, tn = tile.tn;
    const int party = pb / g.batch, b = pb % g.batch;

    // fragment streams: step < ktn uses (E, B_i'), step >= ktn uses (A_i, F)
    const size_t slotA = (size_t)g.batch * g.nblkA * g.KT * (kDigits * kFrag);
    const size_t slotB = (size_t)g.batch * g.nblkB * g.KT * (kDigits * kFrag);
    const char *a_first = g.packA + (size_t)b * g.nblkA * g.KT * (kDigits * kFrag);   // E
    const char *a_second = a_first + (size_t)(1 + party) * slotA;                      // A_i
    const char *b_second = g.packB + (size_t)b * g.nblkB * g.KT * (kDigits * kFrag);  // F
    const char *b_first = b_second + (size_t)(1 + party) * slotB;                      // B_i'

    // this workgroup's k-steps [s0, s0 + steps) of the 2 * ktn (both counts even)
    const int s0 = split * g.split_steps;
    const int steps = min(g.split_steps, 2 * g.ktn - s0);
    const bool starts_in_second = s0 >= g.ktn;
    const u32 lds0 = (u32)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
    const u32 lane16 = lane * 16;

    // Load cursor: where the loads of the next step to be fetched come from and go to.  It lives on
    // the scalar unit and advances by one k-tile per step (no division, no per-load selects); at the
    // switch from the first operand pair to the second it jumps to the other fragment streams.
    // This wave loads fragments f = 4q + wave, q < loads_per_wave: row/column block f / ND = q / (ND/4)
    // of the tile and digit f % ND = 4 (q % (ND/4)) + wave, so only q-dependent constants remain per load.
    const size_t blk_stride = (size_t)g.KT * (kDigits * kFrag);
    const size_t kt0_off = (size_t)g.kt0 * (kDigits * kFrag) + wave * kFrag;
    const char *second_a = a_second + (size_t)tm * (S::BM / 32) * blk_stride + kt0_off;
    const char *second_b = b_second + (size_t)tn * (S::BN / 32) * blk_stride + kt0_off;
    const size_t start_off = (size_t)(starts_in_second ? s0 - g.ktn : s0) * (kDigits * kFrag);
    const char *ld_a = (starts_in_second ? second_a : a_first + (size_t)tm * (S::BM / 32) * blk_stride + kt0_off) + start_off;
    const char *ld_b = (starts_in_second ? second_b : b_first + (size_t)tn * (S::BN / 32) * blk_stride + kt0_off) + start_off;
    int ld_left = starts_in_second ? 0x7fffffff : g.ktn - s0;   // steps until the cursor switches operand pair
    u32 ld_lds = lds0 + wave * kFrag;                    // LDS destination of the cursor's stage
    const u32 lds_wrap = lds0 + wave * kFrag + (S::NSTAGE - 1) * S::stage_bytes;
    auto issue_load = [&](int q) {                       // q is a compile-time constant after unrolling
        constexpr int qa = S::FA / 4;                    // loads of left-operand fragments per wave
        constexpr int per_blk = kDigits / 4;             // loads of this wave per 32-row (32-column) block
        const char *p = q < qa ? ld_a + (size_t)(q / per_blk) * blk_stride + (q % per_blk) * (4 * kFrag)
                               : ld_b + (size_t)((q - qa) / per_blk) * blk_stride + ((q - qa) % per_blk) * (4 * kFrag);
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
                        constexpr int rd_every = Ring<T>::rd_every;
                        constexpr int rd_last = rd_every * (S::frags_per_wave - 1);
                        constexpr int ld_first = Ring<T>::ld_first;
                        constexpr int ld_every = Ring<T>::ld_every;
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
    using Y = std::true_type;
    using F = std::false_type;
    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;
    int s = 0;
    for (; s + 4 < steps; s += 2) {                       // steps is even; both halves have all neighbours
        iteration(B0(), Y(), Y(), Y());
        iteration(B1(), Y(), Y(), Y());
    }
    if (steps >= 4) {
        iteration(B0(), Y(), Y(), Y());                   // step steps-4: loads the last step
        iteration(B1(), F(), Y(), Y());
    }
    iteration(B0(), F(), Y(), F());                       // step steps-2

    // C_i is fetched under the last step (the fragment buffer that step would have filled is free), so that
    // the epilogue starts with its operands at hand instead of a memory round trip with nothing else on the
    // CU.  Rows and columns beyond the matrix are redirected to its last row / column; what they bring is
    // never stored.  C and Z may be the same buffer: every element is read and written by the same lane.
    // With several workgroups per tile (splits > 1) Z already holds C and every part is added atomically:
    // ring addition is associative and commutative, so the result does not depend on the order of arrival.
    const size_t mat = (size_t)g.M * g.N;
    const T *Cm = g.C + (size_t)pb * mat;
    T *Zm = g.Z + (size_t)pb * mat;
    const bool interior = (tm + 1) * S::BM <= g.M && (tn + 1) * S::BN <= g.N;     // uniform over the workgroup
    const bool atomic = g.splits > 1;
    T cv[WM][WN][16];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int col = min(tn * S::BN + (wn * WN + j) * 32 + lane % 32, g.N - 1);
            const int row0 = tm * S::BM + (wm * WM + i) * 32 + 4 * (lane / 32);
#pragma unroll
            for (int r = 0; r < 16; ++r)
                cv[i][j][r] = atomic ? (T)0 : Cm[(size_t)min(row0 + 8 * (r / 4) + r % 4, g.M - 1) * g.N + col];
        }
    __builtin_amdgcn_sched_barrier(0);
    iteration(B1(), F(), F(), F());                       // step steps-1

    // Recombine the diagonals and add C_i.
    // Tiles that lie wholly inside the matrix take branch-free stores: with a bounds check per element every
    // store sits in a basic block of its own and waits for the one before.
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) {                   // one 32 x 32 MFMA tile at a time
            const int col = tn * S::BN + (wn * WN + j) * 32 + lane % 32;
            const int row0 = tm * S::BM + (wm * WM + i) * 32 + 4 * (lane / 32);
            auto row_of = [&](int r) { return row0 + 8 * (r / 4) + r % 4; };
            T v[16];
            __builtin_amdgcn_sched_barrier(0);           // keeps the scheduler from hoisting the next tile's work
#pragma unroll
            for (int r = 0; r < 16; ++r) v[r] = cv[i][j][r];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if constexpr (kDigits == 8)
                    v[r] += recombine_diagonals(acc[i][j][0][r], acc[i][j][1][r], acc[i][j][2][r], acc[i][j][3][r],
                                                acc[i][j][4 % kDigits][r], acc[i][j][5 % kDigits][r],
                                                acc[i][j][6 % kDigits][r], acc[i][j][7 % kDigits][r]);
                else
                    v[r] += recombine_diagonals(acc[i][j][0][r], acc[i][j][1][r], acc[i][j][2][r], acc[i][j][3][r]);
            }
            if (atomic) {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (interior || (row_of(r) < g.M && col < g.N)) ring_atomic_add(Zm + (size_t)row_of(r) * g.N + col, v[r]);
            } else if (interior) {
#pragma unroll
                for (int r = 0; r < 16; ++r) Zm[(size_t)row_of(r) * g.N + col] = v[r];
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (row_of(r) < g.M && col < g.N) Zm[(size_t)row_of(r) * g.N + col] = v[r];
            }
        }
}

template <class T>
__global__ __launch_bounds__(256) void limb_gemm_kernel(GemmArgs<T> g)
{
    limb_gemm_body<T>(g, blockIdx.x);
}

// Products of different shapes in one launch (the grouped call): every workgroup finds its product in the table.
template <class T>
__global__ __launch_bounds__(256) void limb_gemm_grouped_kernel(GroupTable<GemmArgs<T>> t)
{
    const int gi = group_of(t, blockIdx.x);
    limb_gemm_body<T>(t.e[gi], blockIdx.x - t.first[gi]);
}

// ------------------------------------------------- row-streaming GEMM ---
// Z_2^64 products whose output is a single column tile (N <= 64): every left fragment would be used by
// exactly one output tile, so writing the left operands out as fragments and reading them back (the pack
// pre-pass) costs more HBM traffic than the product itself.  Here the left fragments never exist in
// memory.  (Products of a few column tiles and a short inner dimension -- the attention shapes -- take the
// same kernel once per column tile when that is cheaper than the pre-pass: the raw tiles are then read once
// per column tile, from L2.)  One workgroup owns a block of 32 rows and one column tile of 64 for ALL
// parties (NP <= 3) and walks the inner dimension once; the raw 32 x 32 tiles of every X_j and A_j go memory -> LDS exactly once (direct-to-LDS loads,
// no register is held while they fly).
//   producer wave (the last one, on a SIMD of its own)  issues those loads one k-tile ahead, opens
//       E = sum_j (X_j - A_j) from the raw tiles, converts E to digits and lays it out as MFMA fragments
//       in a two-stage LDS ring;
//   consumer wave p (one per party, each with the whole accumulator file)  computes
//       Z_p[32 x 64] = C_p + A_p . F + E . B_p': per 32-deep k-tile a half step on (A_p, F) and one on
//       (E, B_p'), 72 MFMAs each.  It converts its own A_p from the raw tile in registers (the vector ALU is
//       idle under the MFMAs) and reads the right fragments (packed beforehand: they are small, shared by
//       all row blocks and stay in L2) straight from memory into registers, because B_p' has no second
//       reader inside the workgroup.
// Nothing is masked at ragged edges: loads that would leave the matrix are redirected to the tile's first
// element, and what they bring only meets zero-padded rows of the right fragments (k >= K) or lands in
// output rows that are never stored (row >= M).
// Synchronisation: one workgroup barrier per k-tile.  In iteration g the consumers read E(g) from ring
// stage g % 2 (first half) and raw A_p(g+1) from raw slot (g+1) % 3 (second half); the producer reads raw
// slot (g+1) % 3, writes E(g+1) to stage (g+1) % 2, refills raw slot g % 3 with k-tile g + 3 and waits for
// k-tile g + 2, issued one iteration earlier: every load has two iterations to arrive.
// A launch has at most one workgroup per CU (more would only queue: a workgroup takes a whole CU); each walks
// its share of the (row block, column tile) items, and g above counts the k-tiles of all its items in one
// sequence: the producer runs ahead across item boundaries, so that the first tiles of the next item arrive
// and its E(0) is opened while the consumers recombine and store the current one.  Two more barriers per item
// frame the consumers' conversion of the item's first A_p tile.
// Workgroups of a row-kernel launch: (row blocks over all batch entries, rounded up to a multiple of 8) x column tiles.
__host__ __device__ inline long rows_grid(int batch, int M, int tilesN)
{
    const long rblocks = (long)batch * ((M + 31) / 32);
    return (rblocks + 7) / 8 * 8 * tilesN;
}

struct RowGemmArgs {
    const u64 *X, *A;        // [n][batch][M][K]
    const char *packB;       // right fragment store [n+1][batch][2 tilesN][KT][8][1024]: slot 0 = F, 1 + i = B_i'
    const u64 *C;            // [n][batch][M][N]
    u64 *Z;
    int batch, M, N, K, KT, tilesN;
};

// Raw tile in LDS: 32 rows of 256 bytes = 16 pieces of 16 bytes (piece 8 h + q = the q-th pair of k of half h);
// piece p of row r sits at position p ^ (r & 15) of its row, so that the 16 lanes that read the same piece of
// 16 consecutive rows hit 16 different 16-byte bank groups of the 256 bytes the LDS serves per cycle (with the
// swizzle over 8 positions only, rows r and r + 8 collided: a two-way conflict on every read).  In group
// terms: the row's two 128-byte halves are swapped when bit 3 of r is set, and piece q sits at position
// q ^ (r & 7) of its half.  A direct-to-LDS load fills 1 KiB = 4 rows x 256 bytes with whole lines of memory.
constexpr int kRawTile = 32 * 32 * 8;
constexpr int kRawSlot = 3 * 2 * kRawTile;               // X_j then A_j for up to three parties
constexpr int kRawSlots = 3;                             // raw k-tiles in LDS: one in use, two in flight
constexpr int kRowLds = kRawSlots * kRawSlot + 2 * 8 * kFrag;    // + two stages of E fragments: all 160 KB of the CU

// 16 direct-to-LDS loads: the 8 chunks of X_j's and A_j's raw tile.  m0 (LDS base of each load) is put
// back afterwards; the scalar add that sets it clobbers scc.
__device__ inline void load_raw_pair(const char *xs, const char *as, u32 lds_dst, const u32 (&voff)[8])
{
    u32 saved_m0;
    asm volatile(
        "s_mov_b32 %0, m0\n\t"
        "s_add_u32 m0, %3, 0x0000\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %4, %1\n\t"
        "s_add_u32 m0, %3, 0x2000\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %4, %2\n\t"
        "s_add_u32 m0, %3, 0x0400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %5, %1\n\t"
        "s_add_u32 m0, %3, 0x2400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %5, %2\n\t"
        "s_add_u32 m0, %3, 0x0800\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %6, %1\n\t"
        "s_add_u32 m0, %3, 0x2800\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %6, %2\n\t"
        "s_add_u32 m0, %3, 0x0c00\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %7, %1\n\t"
        "s_add_u32 m0, %3, 0x2c00\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %7, %2\n\t"
        "s_add_u32 m0, %3, 0x1000\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %8, %1\n\t"
        "s_add_u32 m0, %3, 0x3000\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %8, %2\n\t"
        "s_add_u32 m0, %3, 0x1400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %9, %1\n\t"
        "s_add_u32 m0, %3, 0x3400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %9, %2\n\t"
        "s_add_u32 m0, %3, 0x1800\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %10, %1\n\t"
        "s_add_u32 m0, %3, 0x3800\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %10, %2\n\t"
        "s_add_u32 m0, %3, 0x1c00\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %11, %1\n\t"
        "s_add_u32 m0, %3, 0x3c00\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %11, %2\n\t"
        "s_mov_b32 m0, %0"
        : "=&s"(saved_m0)
        : "s"(xs), "s"(as), "s"(lds_dst), "v"(voff[0]), "v"(voff[1]), "v"(voff[2]), "v"(voff[3]), "v"(voff[4]),
          "v"(voff[5]), "v"(voff[6]), "v"(voff[7])
        : "memory", "scc");
}
static_assert(kRawTile == 0x2000, "load_raw_pair hard-codes the raw tile size");

typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(3))) const u64x2 lds_u64x2;
typedef __attribute__((address_space(3))) const v4i lds_v4i;

template <int NP>
__device__ __forceinline__ void limb_gemm_rows_body(const RowGemmArgs &g, unsigned first_item, unsigned item_stride)
{
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int lane = threadIdx.x % 64;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    // Workgroup ids are dealt round-robin to the 8 XCDs: the column tiles of one block of rows get ids 8 apart,
    // so they meet in one L2 and the raw tiles come from memory once (rows_grid pads the id space to whole
    // groups of 8 row blocks; a workgroup of the padding leaves at once, all four waves together).
    // A workgroup walks the items first_item, first_item + item_stride, ... (the stride is a multiple of 8, so all
    // of them belong to one XCD); the items of the padding have the highest ids, so the valid ones come first.
    const int rblocks = (g.M + 31) / 32;
    // Item i = column tile (i / 8) % tilesN of row block 8 (i / 8 / tilesN) + i % 8 (row blocks counted over all batch
    // entries; all counts are below 2^31, which the host checks).  With x = first_item % 8 the row block is valid
    // while i / (8 tilesN) < ceil((row blocks - x) / 8).
    const unsigned rblocks_all = (unsigned)g.batch * (unsigned)rblocks;
    auto rblock_of = [&](unsigned item) -> unsigned { return item / 8 / (unsigned)g.tilesN * 8 + item % 8; };
    const unsigned x = first_item % 8;
    const unsigned limit = rblocks_all > x ? (rblocks_all - x + 7) / 8 * 8 * (unsigned)g.tilesN : 0;
    const int n_items = first_item < limit ? (int)((limit - 1 - first_item) / item_stride) + 1 : 0;
    if (n_items == 0) return;                            // all four waves together
    const int KT = g.KT;
    lds_char *lds3 = (lds_char *)lds;
    lds_char *e_ring = lds3 + kRawSlots * kRawSlot;
    // this lane's 16 consecutive k of row lane % 32, half lane / 32, in a raw tile: piece q at raw_lane ^ (16 q)
    const u32 raw_lane = (2 * (lane % 32) + (lane / 32 ^ ((lane >> 3) & 1))) * 128 + (lane % 8) * 16;

    if (wave == NP) {
        // ---------------------------------------------------------------- producer
        // load i, lane p: row 4 i + p / 16; its 128-byte slot (p / 8) % 2 holds the half (p / 8) % 2 ^ bit 3 of
        // the row, position p % 8 of it the piece (p % 8) ^ (row & 7); the lane fetches that piece of the row's 256 bytes
        const size_t row_pitch = (size_t)g.K * 8;
        const bool k_edge = KT * 32 > g.K;               // the last k-tile is ragged
        u32 off[8];                                      // per-lane byte offsets from the tile's first element
        u32 k_ok = 0;                                    // bit i: load i of this lane stays inside K in the last k-tile
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = 4 * i + lane / 16, half = ((lane / 8) % 2) ^ ((row >> 3) & 1), piece = (lane % 8) ^ (row & 7);
            off[i] = (u32)(row * row_pitch) + half * 128 + piece * 16;            // K <= 16352: far below 2^32
            if ((KT - 1) * 32 + 16 * half + 2 * piece < g.K) k_ok |= 1u << i;     // K is even
        }
        const size_t party_stride = (size_t)g.batch * g.M * row_pitch;
        const u32 raw0 = (u32)(uintptr_t)lds3;
        // The k-tiles of all items form one sequence t = 0, 1, ..: tile t lives in raw slot t % 3, E(t) in fragment
        // stage t % 2, and the producer runs up to three tiles ahead of the consumers across item boundaries, so
        // the first tiles of the next item arrive, and its E(0) is opened, while the consumers finish this one.
        const int total = n_items * KT;
        unsigned is_item = first_item;                   // issue cursor: item, k-tile within it, raw slot
        int is_k = 0;
        u32 is_slot = 0;
        size_t is_tile0 = 0;
        int is_row0 = 0;
        auto set_issue_item = [&]() {
            const unsigned rblock = rblock_of(is_item);
            is_row0 = (int)(rblock % (unsigned)rblocks) * 32;
            is_tile0 = ((size_t)(rblock / (unsigned)rblocks) * g.M + (size_t)is_row0) * row_pitch;      // party 0, k-tile 0
        };
        set_issue_item();
        auto issue = [&]() {                             // all parties' tiles of the cursor's k-tile -> its raw slot
            const u32 dst = raw0 + is_slot * kRawSlot;
            const bool last = k_edge && is_k + 1 == KT;
            u32 voff[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const bool ok = is_row0 + 4 * i + lane / 16 < g.M && (!last || ((k_ok >> i) & 1));
                voff[i] = ok ? off[i] : 0;
            }
#pragma unroll
            for (int j = 0; j < NP; ++j) {
                const size_t o = is_tile0 + j * party_stride + (size_t)is_k * 256;
                load_raw_pair((const char *)g.X + o, (const char *)g.A + o, dst + j * (2 * kRawTile), voff);
            }
            is_slot = is_slot == kRawSlots - 1 ? 0 : is_slot + 1;
            if (++is_k == KT) {                          // on to the next item (past the last one nothing is issued)
                is_k = 0;
                is_item += item_stride;
                set_issue_item();
            }
        };
        u32 op_slot = 0, op_stage = 0;                   // open cursor
        auto open_tile = [&]() {                         // E of the cursor's tile from its raw slot -> its fragment stage
            lds_char *slot = lds3 + op_slot * kRawSlot;
            u64x2 opened[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) opened[q] = (u64x2)(0);
#pragma unroll
            for (int j = 0; j < NP; ++j)
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const u64x2 xv = *(lds_u64x2 *)(slot + j * (2 * kRawTile) + (raw_lane ^ (16 * q)));
                    const u64x2 av = *(lds_u64x2 *)(slot + j * (2 * kRawTile) + kRawTile + (raw_lane ^ (16 * q)));
                    opened[q] += xv - av;
                }
            u64 w[16];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                w[2 * q] = to_digits<u64>(opened[q].x);
                w[2 * q + 1] = to_digits<u64>(opened[q].y);
            }
            store_digit_rows<u64>(w, lds + kRawSlots * kRawSlot + op_stage * (8 * kFrag) + lane * 16);
            op_slot = op_slot == kRawSlots - 1 ? 0 : op_slot + 1;
            op_stage ^= 1;
        };
        // Two k-tiles are in flight while one is in use.  Loads return in order, so waiting until at most one
        // k-tile's loads (16 NP) are outstanding means that everything older has landed; before a k-tile is
        // issued the count is brought down to 15, which keeps it within the wave's 6-bit counter.
        auto issue_ahead = [&](int t) {                  // issue tile t (if any); on return every older one has landed
            if (t < total) {
                wait_loads<15>();
                issue();
                wait_loads<16 * NP>();
            } else {
                wait_loads<0>();
            }
        };
        issue();
        wait_loads<0>();
        if (total > 1) issue();
        open_tile();
        issue_ahead(2);
        wait_lds();
        int t = 0;
        for (int item = 0; item < n_items; ++item) {
            // before these two: raw tiles t and t + 1 and E(t) are in LDS (from the start-up above or from the
            // last iteration of the item before); between them the consumers take A_p(t) out of its raw slot
            workgroup_barrier();
            workgroup_barrier();
            for (int kt = 0; kt < KT; ++kt, ++t) {       // the barrier that ends iteration t: raw tile t + 2 and E(t + 1) are in LDS
                if (t + 1 < total) open_tile();
                issue_ahead(t + 3);                      // into the slot of tile t, which nobody reads any more
                wait_lds();
                workgroup_barrier();
            }
        }
        return;
    }

    // -------------------------------------------------------------------- consumer
    const int party = wave;
    const u32 lane16 = lane * 16;
    // Right fragments are read with buffer loads: one descriptor per operand (uniform, on the scalar unit),
    // the lane's 16 bytes as the only vector offset, the k-tile and column block in a scalar offset, the
    // digit as the immediate -- so the 32 loads of a k-tile need no per-lane address arithmetic.
    const u32 cb_stride = (u32)KT * (8 * kFrag);         // from column block 0 to column block 1 (< 2^22)
    lds_char *a_raw = lds3 + party * (2 * kRawTile) + kRawTile;      // raw A_p in raw slot 0

    v16i acc[2][8];
    // fragment registers: [0..15] right (column block q / 8, digit q % 8), [16..23] left (digit q - 16);
    // buffer 0 serves the (E, B_p') half step, buffer 1 the (A_p, F) half step
    v4i fr[2][24];
    auto right_fragment = [&](int q, __amdgpu_buffer_rsrc_t rsrc, u32 koff) -> v4i {
        const u32 soff = koff + (q / 8) * cb_stride + (q % 8 >= 4 ? 4 * kFrag : 0);
        return (v4i)__builtin_amdgcn_raw_buffer_load_b128(rsrc, lane16 + (q % 4) * kFrag, soff, 0);
    };
    // A_p from the raw tile to the eight left fragments of buffer 1, a quarter (elements 4 c .. 4 c + 3 of this
    // lane's 16 = pieces 2 c, 2 c + 1 -> component c of every fragment) at a time, in steps small enough to
    // sit between two MFMAs without holding the matrix pipe up:
    //   step 0  read the two pieces from LDS          step 1, 2  balanced digits of elements 0, 1 / 2, 3
    //   step 3..6  the 4 x 4 byte transposes of the low / high words: first level, second level
    u64x2 piece[2];
    u64 dig[4];
    u32 half_t[4];
    auto convert_step = [&](int c, int step, lds_char *tile) {
        if (step == 0) {
            piece[0] = *(lds_u64x2 *)(tile + (raw_lane ^ (32 * c)));
            piece[1] = *(lds_u64x2 *)(tile + (raw_lane ^ (32 * c + 16)));
        } else if (step == 1) {
            dig[0] = to_digits<u64>(piece[0].x);
            dig[1] = to_digits<u64>(piece[0].y);
        } else if (step == 2) {
            dig[2] = to_digits<u64>(piece[1].x);
            dig[3] = to_digits<u64>(piece[1].y);
        } else {
            const int word = (step - 3) / 2;
            if ((step - 3) % 2 == 0) {
                const u32 a0 = (u32)(dig[0] >> (32 * word)), a1 = (u32)(dig[1] >> (32 * word));
                const u32 a2 = (u32)(dig[2] >> (32 * word)), a3 = (u32)(dig[3] >> (32 * word));
                half_t[0] = __builtin_amdgcn_perm(a1, a0, 0x05010400u);
                half_t[1] = __builtin_amdgcn_perm(a1, a0, 0x07030602u);
                half_t[2] = __builtin_amdgcn_perm(a3, a2, 0x05010400u);
                half_t[3] = __builtin_amdgcn_perm(a3, a2, 0x07030602u);
            } else {
                fr[1][16 + 4 * word + 0][c] = (int)__builtin_amdgcn_perm(half_t[2], half_t[0], 0x05040100u);
                fr[1][16 + 4 * word + 1][c] = (int)__builtin_amdgcn_perm(half_t[2], half_t[0], 0x07060302u);
                fr[1][16 + 4 * word + 2][c] = (int)__builtin_amdgcn_perm(half_t[3], half_t[1], 0x05040100u);
                fr[1][16 + 4 * word + 3][c] = (int)__builtin_amdgcn_perm(half_t[3], half_t[1], 0x07060302u);
            }
        }
    };
    // One half step of 72 MFMAs on buffer CUR; between them the other buffer is filled for the half step
    // that follows.  After the even MFMAs 0, 2, .. 30: its 16 right fragments (memory).  Its left fragments:
    // E from the fragment ring (8 LDS reads after the even MFMAs 32 .. 46, CUR = 1), or A_p converted from the
    // raw tile (CUR = 0): conversion step m = 0 .. 25 after the odd MFMA 2 m + 1, quarter c reading at
    // m = 6 c - 1 (0 for c = 0) and working at m = 6 c + 2 .. 6 c + 7.  sched_barrier pins the interleave.
    auto half_step = [&](auto cur_c, auto fill_c, __amdgpu_buffer_rsrc_t rsrc, u32 koff, lds_char *left) {
        constexpr int cur = decltype(cur_c)::value, nxt = cur ^ 1;
        constexpr bool FILL = decltype(fill_c)::value;
        int slot = 0;
#pragma unroll
        for (int da = 0; da < 8; ++da)
#pragma unroll
            for (int db = 0; db + da < 8; ++db)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    acc[j][da + db] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fr[cur][16 + da], fr[cur][8 * j + db],
                                                                            acc[j][da + db], 0, 0, 0);
                    if (FILL && slot % 2 == 0) {
                        const int item = slot / 2;
                        if (item < 16) {
                            fr[nxt][item] = right_fragment(item, rsrc, koff);
                            __builtin_amdgcn_sched_barrier(0);
                        } else if (cur == 1 && item < 24) {
                            fr[0][item] = *(lds_v4i *)(left + lane16 + (item - 16) * kFrag);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
                    if (FILL && cur == 0 && slot % 2 == 1) {
                        const int m = slot / 2;
                        if (m == 0) convert_step(0, 0, left);
                        if (m >= 5 && m <= 17 && (m + 1) % 6 == 0) convert_step((m + 1) / 6, 0, left);
                        if (m >= 2 && m <= 25) convert_step((m - 2) / 6, 1 + (m - 2) % 6, left);
                        if (m <= 25) __builtin_amdgcn_sched_barrier(0);
                    }
                    ++slot;
                }
    };
    using Y = std::true_type;
    using F = std::false_type;
    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;

    u32 par = 0;                                         // t % 2 and t % 3 of the current tile of the workgroup's sequence
    u32 slot = 0;
    unsigned item_id = first_item;
    for (int item = 0; item < n_items; ++item, item_id += item_stride) {
    const int tn = (int)(item_id / 8 % (unsigned)g.tilesN);
    const unsigned rblock = rblock_of(item_id);
    const int rb = (int)(rblock % (unsigned)rblocks), b = (int)(rblock / (unsigned)rblocks);
    const char *f_base = g.packB + ((size_t)b * g.tilesN + tn) * 2 * cb_stride;                              // F
    const char *b_base = g.packB + (((size_t)(1 + party) * g.batch + b) * g.tilesN + tn) * 2 * cb_stride;    // B_p'
    const __amdgpu_buffer_rsrc_t f_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)f_base, 0, 2 * cb_stride, 0x00020000);
    const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)b_base, 0, 2 * cb_stride, 0x00020000);
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int d = 0; d < 8; ++d) acc[j][d] = (v16i)(0);
#pragma unroll
    for (int q = 0; q < 16; ++q) fr[1][q] = right_fragment(q, f_rsrc, 0);   // in flight while the producer starts up
    workgroup_barrier();                                 // raw tiles t and t + 1 and E(t) are in LDS
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int step = 0; step < 7; ++step) convert_step(c, step, a_raw + slot * kRawSlot);
    wait_lds();
    workgroup_barrier();                                 // the raw slot of tile t may be refilled
    u32 koff = 0;                                        // byte offset of the current k-tile in a fragment stream
    for (int kt = 0; kt + 1 < KT; ++kt) {                // the last k-tile is peeled: no branch around MFMAs
        half_step(B1(), Y(), b_rsrc, koff, e_ring + par * (8 * kFrag));                // A_p . F; fills (E, B_p') of kt
        koff += 8 * kFrag;
        par ^= 1;
        slot = slot == kRawSlots - 1 ? 0 : slot + 1;
        half_step(B0(), Y(), f_rsrc, koff, a_raw + slot * kRawSlot);                    // E . B_p'; fills (A_p, F) of kt + 1
        wait_lds();
        workgroup_barrier();
    }
    koff = (u32)(KT - 1) * (8 * kFrag);                  // restated from the argument, so that it stays scalar
    half_step(B1(), Y(), b_rsrc, koff, e_ring + par * (8 * kFrag));

    // C_p is fetched under the last half step (the fragment buffer that half step would have filled is free):
    // the epilogue then starts with its operands at hand.  Rows and columns beyond the matrix are redirected
    // to its last row / column; what they bring is never stored.  C may be Z itself: every element is read
    // and written by the same lane of the same workgroup.
    const size_t zmat = (size_t)g.M * g.N;
    const u64 *Cm = g.C + ((size_t)party * g.batch + b) * zmat;
    u64 *Zm = g.Z + ((size_t)party * g.batch + b) * zmat;
    const bool interior = (rb + 1) * 32 <= g.M && (tn + 1) * 64 <= g.N;
    const int row0 = rb * 32 + 4 * (lane / 32);
    auto row_of = [&](int r) { return row0 + 8 * (r / 4) + r % 4; };
    u64 cv[2][16];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int col = min(tn * 64 + j * 32 + lane % 32, g.N - 1);
#pragma unroll
        for (int r = 0; r < 16; ++r) cv[j][r] = Cm[(size_t)min(row_of(r), g.M - 1) * g.N + col];
    }
    __builtin_amdgcn_sched_barrier(0);
    half_step(B0(), F(), f_rsrc, koff, a_raw);
    workgroup_barrier();
    par ^= 1;                                            // past the item's last tile
    slot = slot == kRawSlots - 1 ? 0 : slot + 1;

    // recombine the diagonals, add C_p, store (same structure as the tile kernel's epilogue)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int col = tn * 64 + j * 32 + lane % 32;
        u64 v[16];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] = cv[j][r];
#pragma unroll
        for (int r = 0; r < 16; ++r)
            v[r] += recombine_diagonals(acc[j][0][r], acc[j][1][r], acc[j][2][r], acc[j][3][r], acc[j][4][r], acc[j][5][r],
                                        acc[j][6][r], acc[j][7][r]);
        if (interior) {
#pragma unroll
            for (int r = 0; r < 16; ++r) Zm[(size_t)row_of(r) * g.N + col] = v[r];
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (row_of(r) < g.M && col < g.N) Zm[(size_t)row_of(r) * g.N + col] = v[r];
        }
    }
    }                                                    // next item
}

template <int NP>
__global__ __launch_bounds__(64 * (NP + 1)) void limb_gemm_rows_kernel(RowGemmArgs g)
{
    limb_gemm_rows_body<NP>(g, blockIdx.x, gridDim.x);
}

template <int NP>
__global__ __launch_bounds__(64 * (NP + 1)) void limb_gemm_rows_grouped_kernel(GroupTable<RowGemmArgs> t)
{
    const int gi = group_of(t, blockIdx.x);
    limb_gemm_rows_body<NP>(t.e[gi], blockIdx.x - t.first[gi], 0x7fffffffu);
}

// ------------------------------------------------------------------ host ---
struct Plan {
    int KT, nblkA, nblkB, tilesM, tilesN;
    size_t packA_bytes, packB_bytes;
};
template <class T> inline Plan make_plan(int n, int batch, int M, int N, int K)
{
    using S = GemmShape<T>;
    Plan p;
    p.KT = ceil_div(K, 32);
    p.tilesM = ceil_div(M, S::BM);
    p.tilesN = ceil_div(N, S::BN);
    p.nblkA = p.tilesM * (S::BM / 32);
    p.nblkB = p.tilesN * (S::BN / 32);
    p.packA_bytes = (size_t)(n + 1) * batch * p.nblkA * p.KT * (S::ND * kFrag);
    p.packB_bytes = (size_t)(n + 1) * batch * p.nblkB * p.KT * (S::ND * kFrag);
    return p;
}

// How many workgroups share one output tile.  One workgroup per CU is resident at a time, so `tiles`
// tiles of `steps` k-steps take ceil(tiles / CUs) rounds of steps + a fixed prologue/epilogue cost; when
// the tiles do not fill the chip, splitting the k-steps of each tile over several workgroups (which add
// their parts onto Z atomically) shortens the rounds.  Returns the count that minimises that model.
inline int choose_splits(long tiles, int steps)
{
    const int cus = compute_units();
    constexpr int kFixedCost = 8;                        // prologue + epilogue, in k-step equivalents
    constexpr int kMinSteps = 8;                         // shorter parts are all overhead
    long best_cost = -1;
    int best = 1;
    for (int sp = 1; sp <= 16; ++sp) {
        const int part = 2 * ceil_div(ceil_div(steps, 2), sp);
        if (sp > 1 && part < kMinSteps) break;
        const long rounds = (tiles * sp + cus - 1) / cus;
        const long cost = rounds * (part + kFixedCost);
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = sp; }
    }
    return best;
}

// Whether the row-streaming kernel takes a product: 64-bit ring, at most three parties (one consumer wave
// each), even K (16-byte row alignment), an inner dimension one launch may accumulate, and a lower
// estimated cost than the tile kernel plus its pre-pass over the left operands.  Costs are in k-steps of
// one CU (about a microsecond), the unit of choose_splits: the row kernel walks 2 KT steps per block of 32
// rows and column tile; the other path adds the left pack, an HBM stream of (3n + 1) operand-sized matrices
// at about 5 MB per step-time, and one more launch.
template <class T> inline bool rows_kernel_applies(const MatmulArgsT<T> &a, const Plan &p)
{
    if (!std::is_same<T, u64>::value) return false;
    if (a.n > 3 || a.K % 2 != 0 || p.KT > Ring<u64>::max_chunk_tiles) return false;
    const int cus = compute_units();
    const long rblocks = rows_grid(a.batch, a.M, p.tilesN);
    if (rblocks > 0x7fffffffL) return false;
    const double cost_rows = (double)((rblocks + cus - 1) / cus) * (2 * p.KT + 8);
    const long tiles = (long)p.tilesM * p.tilesN * a.n * a.batch;
    const int sp = choose_splits(tiles, 2 * p.KT);
    const double pack_bytes = 8.0 * (3 * a.n + 1) * a.batch * (double)a.M * a.K;
    const double cost_tiles = (double)((tiles * sp + cus - 1) / cus) * (2 * ceil_div(p.KT, sp) + 8) + pack_bytes / 5.0e6 + 5;
    return cost_rows <= cost_tiles;
}

inline spin_status launch_rows(const MatmulArgs &a, const Plan &p, char *packB, hipStream_t s, const char *where_pack,
                               const char *where_gemm)
{
    {
        KernelTimer timer(SPIN_KERNEL_PACK, s);
        launch_pack_right<u64>(a, packB, p.nblkB, p.KT, s);
        spin_status st = check_launch(where_pack);
        if (st != SPIN_OK) return st;
    }
    RowGemmArgs g{a.X, a.A, packB, a.C, a.Z, a.batch, a.M, a.N, a.K, p.KT, p.tilesN};
    // One workgroup fits a CU, so more workgroups than CUs only queue: launch one per CU (a multiple of 8, so that
    // an item keeps its XCD) and let each walk its items, the producer running ahead across item boundaries.
    const unsigned items = (unsigned)rows_grid(a.batch, a.M, p.tilesN);
    const unsigned resident = (unsigned)std::max(8, compute_units() / 8 * 8);
    const unsigned grid = items > resident && ((long)items / resident + 1) * p.KT < (1L << 30) ? resident : items;
    spin_status st = SPIN_OK;
    for_party_count(a.n, [&](auto np) {
        constexpr int NP = decltype(np)::value <= 3 ? decltype(np)::value : 3;   // n <= 3 is checked by the caller
        static OncePerDevice lds_allowed;
        auto kernel = limb_gemm_rows_kernel<NP>;
        st = allow_dynamic_lds((const void *)kernel, kRowLds, lds_allowed);
        if (st != SPIN_OK) return;
        KernelTimer timer(SPIN_KERNEL_GEMM_LIMB, s);
        kernel<<<grid, 64 * (NP + 1), kRowLds, s>>>(g);
        st = check_launch(where_gemm);
    });
    return st;
}

template <class T> spin_status launch_limb(const MatmulArgsT<T> &a, hipStream_t s, const char *where_pack, const char *where_gemm)
{
    using S = GemmShape<T>;
    const Plan p = make_plan<T>(a.n, a.batch, a.M, a.N, a.K);
    char *packA = (char *)a.workspace;
    char *packB = packA + p.packA_bytes;

    if constexpr (std::is_same<T, u64>::value) {
        if (rows_kernel_applies<T>(a, p)) return launch_rows(a, p, packB, s, where_pack, where_gemm);
    }

    launch_pack<T>(a, packA, packB, p.nblkA, p.nblkB, p.KT, s);
    spin_status st = check_launch(where_pack);
    if (st != SPIN_OK) return st;

    static OncePerDevice lds_allowed;                    // one per ring type
    auto kernel = limb_gemm_kernel<T>;
    st = allow_dynamic_lds((const void *)kernel, S::lds_bytes, lds_allowed);
    if (st != SPIN_OK) return st;
    GemmArgs<T> g{packA, packB, a.C, a.Z, a.n, a.batch, a.M, a.N, p.nblkA, p.nblkB, p.KT, 0, 0, p.tilesM, p.tilesN,
                  1, 0};
    const long total = (long)p.tilesM * p.tilesN * a.n * a.batch;
    constexpr int chunk = Ring<T>::max_chunk_tiles;
    const int first_ktn = p.KT < chunk ? p.KT : chunk;
    const int splits = choose_splits(total, 2 * first_ktn);
    if (splits > 1 && a.C != a.Z) {                      // the parts are added onto Z, which starts out as C
        st = launch_open<T>(a.C, nullptr, (size_t)a.n * a.batch * a.M * a.N, 1, a.Z, s);
        if (st != SPIN_OK) return st;
    }
    for (int kt0 = 0; kt0 < p.KT; kt0 += chunk) {
        g.kt0 = kt0;
        g.ktn = p.KT - kt0 < chunk ? p.KT - kt0 : chunk;
        g.C = kt0 == 0 ? a.C : a.Z;                      // later chunks accumulate onto Z
        g.splits = splits;
        g.split_steps = 2 * ceil_div(g.ktn, splits);     // even, so that every part has an even number of steps
        const int used = ceil_div(2 * g.ktn, g.split_steps);     // parts that actually have steps
        g.splits = used;
        if (splits > 1 && used == 1) g.C = a.Z;          // a short last chunk in one part: plain accumulate onto Z
        KernelTimer timer(SPIN_KERNEL_GEMM_LIMB, s);
        kernel<<<(unsigned)(total * used), 256, S::lds_bytes, s>>>(g);
        st = check_launch(where_gemm);
        if (st != SPIN_OK) return st;
    }
    return SPIN_OK;
}

// ---- grouped call: products of different shapes, a handful of launches for all of them ----------------
// Every group gets its own fragment stores inside the workspace (the packs of all groups run before their
// GEMMs), chooses the row-streaming or the tile kernel as a single product would, and the groups of one kind
// share a launch: right packs (plain / stored transposed), left packs (tile-kernel groups only), row GEMMs,
// tile GEMMs -- at most five launches per kGroupsPerLaunch groups.  Tiles are not shared between workgroups
// here (the groups together fill the chip), so Z needs no pre-copy.
template <class Args, class Launch> inline spin_status launch_in_tables(const std::vector<Args> &args,
                                                                        const std::vector<unsigned> &blocks, Launch &&launch)
{
    for (size_t g0 = 0; g0 < args.size(); g0 += kGroupsPerLaunch) {
        GroupTable<Args> t;
        t.count = (int)std::min<size_t>(kGroupsPerLaunch, args.size() - g0);
        unsigned total = 0;
        for (int i = 0; i < t.count; ++i) {
            t.first[i] = total;
            t.e[i] = args[g0 + i];
            total += blocks[g0 + i];
        }
        for (int i = t.count; i <= kGroupsPerLaunch; ++i) t.first[i] = total;
        launch(t, total);
    }
    return SPIN_OK;
}

}  // namespace

size_t limb_grouped_workspace_bytes(int n, int groups, const MatmulArgs *a)
{
    size_t sum = 0;
    for (int g = 0; g < groups; ++g) sum += limb_workspace_bytes(n, a[g].batch, a[g].M, a[g].N, a[g].K);
    return sum;
}

// Returns SPIN_ERANGE, before anything is launched, when a group cannot go into a shared launch (an inner dimension
// that must be accumulated in several launches, or more workgroups than a grid holds); the caller then enqueues
// the groups one after another.
spin_status launch_matmul_limb_grouped(int n, int groups, const MatmulArgs *a, void *workspace, hipStream_t s)
{
    constexpr int WAVES = 4;
    std::vector<PackArgs<u64>> left, right_plain, right_t;
    std::vector<unsigned> left_blocks, right_plain_blocks, right_t_blocks, row_blocks, tile_blocks;
    std::vector<RowGemmArgs> rows;
    std::vector<GemmArgs<u64>> tiles;
    bool vec = true;
    char *ws = (char *)workspace;
    for (int g = 0; g < groups; ++g) {
        const MatmulArgs &m = a[g];
        const Plan p = make_plan<u64>(n, m.batch, m.M, m.N, m.K);
        if (p.KT > Ring<u64>::max_chunk_tiles) return SPIN_ERANGE;
        vec = vec && m.K % 2 == 0;
        char *packA = ws, *packB = ws + p.packA_bytes;
        ws += p.packA_bytes + p.packB_bytes;
        if (m.y_transposed) {
            right_t.push_back(PackArgs<u64>{m.Y, m.B, packB, n, m.batch, m.N, m.K, p.nblkB, p.KT});
            right_t_blocks.push_back(pack_left_blocks<WAVES>(p.nblkB, p.KT) * m.batch);
        } else {
            right_plain.push_back(PackArgs<u64>{m.Y, m.B, packB, n, m.batch, m.K, m.N, p.nblkB, p.KT});
            right_plain_blocks.push_back(pack_right_blocks(p.nblkB, p.KT) * m.batch);
        }
        if (rows_kernel_applies<u64>(m, p)) {
            rows.push_back(RowGemmArgs{m.X, m.A, packB, m.C, m.Z, m.batch, m.M, m.N, m.K, p.KT, p.tilesN});
            row_blocks.push_back((unsigned)rows_grid(m.batch, m.M, p.tilesN));
        } else {
            left.push_back(PackArgs<u64>{m.X, m.A, packA, n, m.batch, m.M, m.K, p.nblkA, p.KT});
            left_blocks.push_back(pack_left_blocks<WAVES>(p.nblkA, p.KT) * m.batch);
            tiles.push_back(GemmArgs<u64>{packA, packB, m.C, m.Z, n, m.batch, m.M, m.N, p.nblkA, p.nblkB, p.KT, 0, p.KT,
                                          p.tilesM, p.tilesN, 1, 2 * p.KT});
            tile_blocks.push_back((unsigned)((long)p.tilesM * p.tilesN * n * m.batch));
        }
    }
    for (const std::vector<unsigned> *v : {&left_blocks, &right_plain_blocks, &right_t_blocks, &row_blocks, &tile_blocks}) {
        unsigned long sum = 0;                           // a launch of up to kGroupsPerLaunch groups must fit a grid
        for (unsigned b : *v) sum += b;
        if (sum > 0x7fffffffUL) return SPIN_ERANGE;
    }
    spin_status st = SPIN_OK;
    for_party_count(n, [&](auto np) {
        constexpr int NP = decltype(np)::value;
        {
            KernelTimer timer(SPIN_KERNEL_PACK, s);
            launch_in_tables(right_plain, right_plain_blocks, [&](const GroupTable<PackArgs<u64>> &t, unsigned total) {
                pack_right_grouped_kernel<NP, u64, false><<<total, 256, 0, s>>>(t);
            });
            auto pack_rows = [&](const std::vector<PackArgs<u64>> &v, const std::vector<unsigned> &blocks, auto right_c) {
                constexpr bool RIGHT = decltype(right_c)::value;
                launch_in_tables(v, blocks, [&](const GroupTable<PackArgs<u64>> &t, unsigned total) {
                    if (vec) pack_left_grouped_kernel<NP, u64, true, WAVES, RIGHT, false><<<total, 64 * WAVES, 0, s>>>(t);
                    else pack_left_grouped_kernel<NP, u64, false, WAVES, RIGHT, false><<<total, 64 * WAVES, 0, s>>>(t);
                });
            };
            pack_rows(right_t, right_t_blocks, std::true_type());
            pack_rows(left, left_blocks, std::false_type());
            st = check_launch("spin_beaver_matmul_grouped(pack)");
            if (st != SPIN_OK) return;
        }
        if (!rows.empty()) {
            constexpr int RP = NP <= 3 ? NP : 3;             // groups reach the row kernel only when n <= 3
            static OncePerDevice lds_allowed;
            auto kernel = limb_gemm_rows_grouped_kernel<RP>;
            st = allow_dynamic_lds((const void *)kernel, kRowLds, lds_allowed);
            if (st != SPIN_OK) return;
            KernelTimer timer(SPIN_KERNEL_GEMM_LIMB, s);
            launch_in_tables(rows, row_blocks, [&](const GroupTable<RowGemmArgs> &t, unsigned total) {
                kernel<<<total, 64 * (RP + 1), kRowLds, s>>>(t);
            });
            st = check_launch("spin_beaver_matmul_grouped(row gemm)");
            if (st != SPIN_OK) return;
        }
        if (!tiles.empty()) {
            static OncePerDevice lds_allowed;
            auto kernel = limb_gemm_grouped_kernel<u64>;
            st = allow_dynamic_lds((const void *)kernel, GemmShape<u64>::lds_bytes, lds_allowed);
            if (st != SPIN_OK) return;
            KernelTimer timer(SPIN_KERNEL_GEMM_LIMB, s);
            launch_in_tables(tiles, tile_blocks, [&](const GroupTable<GemmArgs<u64>> &t, unsigned total) {
                kernel<<<total, 256, GemmShape<u64>::lds_bytes, s>>>(t);
            });
            st = check_launch("spin_beaver_matmul_grouped(tile gemm)");
        }
    });
    return st;
}

namespace {
}  // namespace

size_t limb_workspace_bytes(int n, int batch, int M, int N, int K)
{
    Plan p = make_plan<u64>(n, batch, M, N, K);
    return p.packA_bytes + p.packB_bytes;
}

size_t limb32_workspace_bytes(int n, int batch, int M, int N, int K)
{
    Plan p = make_plan<u32>(n, batch, M, N, K);
    return p.packA_bytes + p.packB_bytes;
}

spin_status launch_matmul_limb(const MatmulArgs &a, hipStream_t s)
{
    return launch_limb<u64>(a, s, "spin_beaver_matmul(pack)", "spin_beaver_matmul(limb gemm)");
}

spin_status launch_matmul_limb32(const MatmulArgs32 &a, hipStream_t s)
{
    return launch_limb<u32>(a, s, "spin32_beaver_matmul(pack)", "spin32_beaver_matmul(limb gemm)");
}

}  // namespace spin
