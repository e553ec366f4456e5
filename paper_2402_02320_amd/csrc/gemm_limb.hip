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
__global__ __launch_bounds__(256) void limb_gemm_kernel(GemmArgs<T> g)
{
    using S = GemmShape<T>;
    constexpr int kDigits = S::ND, WM = S::WM, WN = S::WN;
    extern __shared__ __attribute__((aligned(1024))) char lds[];

    const int lane = threadIdx.x % 64;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    const int wm = wave / 2, wn = wave % 2;

    // work item = (split, tile), tiles fastest: neighbours on an XCD work on neighbouring tiles of one k-range
    const long tiles_total = (long)g.tilesM * g.tilesN * g.n * g.batch;
    const long item = xcd_contiguous_id(blockIdx.x, tiles_total * g.splits);
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
    iteration(B1(), F(), F(), F());                       // step steps-1

    // Recombine the diagonals and add C_i.  The 16 C values of a lane in one MFMA tile are loaded before
    // the first of its stores: interleaved, every load would wait out the store before it (C and Z may
    // be the same buffer, so the compiler keeps their order), 32 memory round trips in a row with
    // nothing else on the CU.
    // Tiles that lie wholly inside the matrix take branch-free loads and stores: with a bounds check per
    // element every store sits in a basic block of its own and again waits for the one before.  Only
    // the memory accesses are duplicated; the arithmetic between them is shared by both cases.
    const size_t mat = (size_t)g.M * g.N;
    const T *Cm = g.C + (size_t)pb * mat;
    T *Zm = g.Z + (size_t)pb * mat;
    const bool interior = (tm + 1) * S::BM <= g.M && (tn + 1) * S::BN <= g.N;     // uniform over the workgroup
    // With several workgroups per tile (splits > 1) Z already holds C and every part is added atomically:
    // ring addition is associative and commutative, so the result does not depend on the order of arrival.
    const bool atomic = g.splits > 1;
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) {                   // one 32 x 32 MFMA tile at a time
            const int col = tn * S::BN + (wn * WN + j) * 32 + lane % 32;
            const int row0 = tm * S::BM + (wm * WM + i) * 32 + 4 * (lane / 32);
            auto row_of = [&](int r) { return row0 + 8 * (r / 4) + r % 4; };
            T v[16];
            __builtin_amdgcn_sched_barrier(0);           // keeps the scheduler from hoisting the next tile's work
            if (atomic) {
#pragma unroll
                for (int r = 0; r < 16; ++r) v[r] = 0;
            } else if (interior) {
#pragma unroll
                for (int r = 0; r < 16; ++r) v[r] = Cm[(size_t)row_of(r) * g.N + col];
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    v[r] = (row_of(r) < g.M && col < g.N) ? Cm[(size_t)row_of(r) * g.N + col] : (T)0;
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int r = 0; r < 16; ++r)
#pragma unroll
                for (int d = 0; d < kDigits; ++d) v[r] += (T)(int64_t)acc[i][j][d][r] << (8 * d);
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

template <class T> spin_status launch_limb(const MatmulArgsT<T> &a, hipStream_t s, const char *where_pack, const char *where_gemm)
{
    using S = GemmShape<T>;
    const Plan p = make_plan<T>(a.n, a.batch, a.M, a.N, a.K);
    char *packA = (char *)a.workspace;
    char *packB = packA + p.packA_bytes;

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
