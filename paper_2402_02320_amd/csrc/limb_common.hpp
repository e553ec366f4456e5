// What the limb-decomposed GEMMs over Z_2^32, Z_2^64 and Z_2^128 share: the balanced-digit conversion, the
// fragment layout and the two pack kernels that open E (F) and lay all left (right) operands out as
// int8 MFMA fragments, the direct-to-LDS load, and the mapping of workgroup ids to output tiles.
//
// A ring element of ND bytes (ND = 4, 8 or 16) is rewritten as ND balanced digits s_i in [-128,127] with
// sum_i s_i 256^i == a (mod 2^(8 ND)):  t = a + 0x80..80;  s = t ^ 0x80..80 (bytes read as int8).
// Fragment store: [slot][batch][blk][kt][digit][1024 B]; in one 1 KiB fragment lane l's 16 bytes at
// offset 16 l are digit d of elements (row or column 32 blk + l % 32, k = 32 kt + 16 (l / 32) + 0..15),
// which is exactly one operand of v_mfma_i32_32x32x32_i8.  Zero padded to whole tiles.
#pragma once
#include "common.hpp"

namespace spin {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kFrag = 1024;          // bytes of one 32x32 int8 fragment

template <class T> __device__ inline T digit_bias();
template <> __device__ inline u32 digit_bias<u32>() { return 0x80808080u; }
template <> __device__ inline u64 digit_bias<u64>() { return 0x8080808080808080ull; }
template <> __device__ inline u128 digit_bias<u128>()
{
    return ((u128)0x8080808080808080ull << 64) | 0x8080808080808080ull;
}
template <class T> __device__ inline T to_digits(T a) { return (a + digit_bias<T>()) ^ digit_bias<T>(); }

// Transposes 16 digit-words (16 elements x ND digits) into ND rows of 16 bytes and stores row p
// (digit p of the 16 elements) at dst + p*kFrag; NT: with non-temporal stores.
template <class T, bool NT = false> __device__ inline void store_digit_rows(const T (&w)[16], char *dst)
{
#pragma unroll
    for (int word = 0; word < (int)sizeof(T) / 4; ++word) {     // digits 4 word .. 4 word + 3
        u32 rows[4][4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            u32 w0 = (u32)(w[4 * q + 0] >> (32 * word)), w1 = (u32)(w[4 * q + 1] >> (32 * word));
            u32 w2 = (u32)(w[4 * q + 2] >> (32 * word)), w3 = (u32)(w[4 * q + 3] >> (32 * word));
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
            if constexpr (NT) __builtin_nontemporal_store(v, (v4i *)(dst + (size_t)(word * 4 + p) * kFrag));
            else *(v4i *)(dst + (size_t)(word * 4 + p) * kFrag) = v;
        }
    }
}

// Operand sets far larger than the caches are read once and their fragments written once: the pack kernels
// then use non-temporal loads and stores (NT), measured 7 % faster at 5 parties x 4096^2 per side; smaller
// calls keep ordinary accesses so that the GEMM finds the fragments in L2.
constexpr size_t kPackStreamingBytes = (size_t)64 << 20;
template <bool NT, class T> __device__ inline T load_share(const T *p)
{
    if constexpr (NT && sizeof(T) == 8) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT> __device__ inline u64x2 load_share_pair(const u64 *p)
{
    if constexpr (NT) return __builtin_nontemporal_load((const u64x2 *)p);
    else return *(const u64x2 *)p;
}

template <class T> struct PackArgs {
    const T *val;       // X or Y shares   [n][batch][rows][cols]
    const T *tri;       // A or B shares   [n][batch][rows][cols]
    char *pack;         // [n+1][batch][nblk][KT][ND][1024]
    int n, batch;
    int rows, cols;     // source matrix is rows x cols, row-major
    int nblk, KT;       // blocks of 32 along the non-contracted axis; k-tiles of 32
};

// Both pack kernels make one pass over the 2n share streams of their side: the opened matrix (E or F)
// accumulates in registers while each triple share is converted and stored as it arrives.  Slots:
// 0 = opened, 1 + i = party i's triple share (left side A_i; right side B_i, and for party 0 B_0 + F,
// which folds the public E.F term into party 0's first product).  blockIdx.z = batch.  Party 0's triple share is needed again at the end (B_0 + F): rings of
// up to 8 bytes keep it in registers, 16-byte rings read it a second time (KEEP = false) to stay within
// the register file.

// Right side: source K x N row-major, a fragment row is a matrix column, so the 16 consecutive k a
// lane needs are 16 strided loads whose lanes run along contiguous columns.  One wave handles 64
// columns x 16 k (half a k-tile of two adjacent column blocks): every wave-wide load is one contiguous
// 64-element row segment, every store two contiguous half-fragment chunks; consecutive waves continue
// along the row.
// `block` is the workgroup's index within its batch entry b.
template <int NP, class T, bool NT>
__device__ __forceinline__ void pack_right_body(const PackArgs<T> &a, long block, int b)
{
    constexpr int ND = sizeof(T);
    constexpr bool KEEP = sizeof(T) <= 8;
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int nblk2 = (a.nblk + 1) / 2;                    // pairs of column blocks
    const long tile = block * 4 + wave;                    // (kt, half, block pair), block pair fastest
    if (tile >= (long)nblk2 * a.KT * 2) return;
    const int blk2 = (int)(tile % nblk2);
    const int half = (int)(tile / nblk2 % 2), kt = (int)(tile / nblk2 / 2);
    const int blk = blk2 * 2 + lane / 32;
    const int K = a.rows, N = a.cols;
    const int col = blk2 * 64 + lane;
    const int k0 = kt * 32 + 16 * half;
    const bool owns = blk < a.nblk;                        // the last pair may have only one block
    const size_t mat = (size_t)K * N;
    const size_t party_stride = (size_t)a.batch * mat;
    auto frag = [&](int slot) -> char * {
        return a.pack + ((((size_t)slot * a.batch + b) * a.nblk + blk) * a.KT + kt) * (ND * kFrag) +
               (lane % 32 + 32 * half) * 16;
    };
    T opened[16], first[KEEP ? 16 : 1];
#pragma unroll
    for (int j = 0; j < 16; ++j) opened[j] = 0;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        const T *v = a.val + (size_t)i * party_stride + (size_t)b * mat;
        const T *t = a.tri + (size_t)i * party_stride + (size_t)b * mat;
        // Loads are unconditional (an out-of-range element reads element 0 and is replaced by zero):
        // guarded by a branch each, every load would be awaited before the next one is issued.
        T tv[16], xv[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const bool ok = col < N && k0 + j < K;
            const size_t e = ok ? (size_t)(k0 + j) * N + col : 0;
            tv[j] = load_share<NT>(t + e);
            xv[j] = load_share<NT>(v + e);
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const bool ok = col < N && k0 + j < K;
            tv[j] = ok ? tv[j] : (T)0;
            opened[j] += ok ? xv[j] - tv[j] : (T)0;
        }
        if (i == 0) {
            if (KEEP) {
#pragma unroll
                for (int j = 0; j < 16; ++j) first[j] = tv[j];
            }
        } else {
#pragma unroll
            for (int j = 0; j < 16; ++j) tv[j] = to_digits<T>(tv[j]);
            if (owns) store_digit_rows<T, NT>(tv, frag(i + 1));
        }
    }
    T w[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) w[j] = to_digits<T>(opened[j]);
    if (owns) store_digit_rows<T, NT>(w, frag(0));
    const T *t0 = a.tri + (size_t)b * mat;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        T f0 = 0;
        if (KEEP) {
            f0 = first[j];
        } else {
            const bool ok = col < N && k0 + j < K;
            f0 = t0[ok ? (size_t)(k0 + j) * N + col : 0];
            f0 = ok ? f0 : (T)0;
        }
        w[j] = to_digits<T>(f0 + opened[j]);
    }
    if (owns) store_digit_rows<T, NT>(w, frag(1));
}
__host__ __device__ inline unsigned pack_right_blocks(int nblk, int KT) { return (unsigned)(((long)((nblk + 1) / 2) * KT * 2 + 3) / 4); }

template <int NP, class T, bool NT>
__global__ __launch_bounds__(256) void pack_right_kernel(PackArgs<T> a)
{
    pack_right_body<NP, T, NT>(a, blockIdx.x, blockIdx.z);
}

// Several products of different shapes in one launch (the grouped call): the descriptors travel as a kernel
// argument, every workgroup looks its group up from the table of first workgroup ids.
constexpr int kGroupsPerLaunch = 32;
template <class Args> struct GroupTable {
    int count;
    unsigned first[kGroupsPerLaunch + 1];                  // first workgroup id of every group, then the total
    Args e[kGroupsPerLaunch];
};
template <class Args> __device__ inline int group_of(const GroupTable<Args> &t, unsigned id)
{
    int g = 0;
    for (int i = 1; i < t.count; ++i) g += id >= t.first[i] ? 1 : 0;
    return g;
}

template <int NP, class T, bool NT>
__global__ __launch_bounds__(256) void pack_right_grouped_kernel(GroupTable<PackArgs<T>> t)
{
    const int gi = group_of(t, blockIdx.x);
    const PackArgs<T> a = t.e[gi];
    const unsigned local = blockIdx.x - t.first[gi], per_batch = pack_right_blocks(a.nblk, a.KT);
    pack_right_body<NP, T, NT>(a, local % per_batch, (int)(local / per_batch));
}

// Left side: source M x K row-major, a fragment row is a matrix row.  Reading 16 consecutive k per
// lane directly would make every wave-wide load touch 64 different rows; instead a wave reads its
// 32 x 32 tile (blk, kt) as whole-row segments (16 bytes per lane, 32 k of one row contiguous), sums the parties'
// shares in that layout, and turns each 32 x 32 tile through LDS (rows padded by 16 bytes,
// conflict-free for 16-byte accesses both ways) so that each lane ends up with the 16 consecutive k
// of one row that a fragment chunk needs.  WAVES = waves per block (LDS: WAVES x 32 padded rows).
// RIGHT = true packs a right operand that is stored transposed ([N][K] row-major, the layout of K in
// Q.K^T): the access pattern is the left side's, the slot rule the right side's (party 0's slot holds
// B_0 + F).
template <int NP, class T, bool VEC, int WAVES, bool RIGHT, bool NT>
__device__ __forceinline__ void pack_left_body(const PackArgs<T> &a, long block, int b)
{
    constexpr int ND = sizeof(T);
    constexpr bool KEEP = sizeof(T) <= 8;
    constexpr int EPL = 16 / ND;                 // elements per 16-byte lane load: 4, 2 or 1
    constexpr int LPR = 32 / EPL;                // lanes that cover the 32 k of one row: 8, 16 or 32
    constexpr int RPL = 64 / LPR;                // rows per wave-wide load: 8, 4 or 2
    constexpr int NL = 32 / RPL;                 // loads per lane: 4, 8 or 16
    constexpr int kRowBytes = 32 * ND + 16;
    struct alignas(16) Pair { T e[EPL]; };
    __shared__ __attribute__((aligned(16))) char turn[WAVES][32 * kRowBytes];
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    long tile = block * WAVES + wave;                       // (blk, kt) pair
    const bool active = tile < (long)a.nblk * a.KT;
    if (!active) tile = 0;
    const int blk = (int)(tile / a.KT), kt = (int)(tile % a.KT);
    const int M = a.rows, K = a.cols;
    const size_t mat = (size_t)M * K;
    const size_t party_stride = (size_t)a.batch * mat;
    const int kk = kt * 32 + EPL * (lane % LPR);            // this lane's k (pair) of every row it loads
    auto frag = [&](int slot) -> char * {
        return a.pack + ((((size_t)slot * a.batch + b) * a.nblk + blk) * a.KT + kt) * (ND * kFrag) + lane * 16;
    };
    // elements (row, kk ..), zero outside.  The loads themselves are unconditional (an out-of-range
    // element reads element 0 of the matrix and is replaced by zero), so that none of them sits behind
    // a branch and has to be awaited before the next is issued.
    auto load = [&](const T *base, int row) -> Pair {
        Pair v;
        if (VEC) {
            const bool ok = row < M && kk < K;
            const T *src = base + (ok ? (size_t)row * K + kk : 0);
            if constexpr (NT && sizeof(T) == 8) {
                const u64x2 two = load_share_pair<true>((const u64 *)src);
                v.e[0] = two.x;
                v.e[1] = two.y;
            } else {
                v = *(const Pair *)src;
            }
#pragma unroll
            for (int q = 0; q < EPL; ++q) v.e[q] = ok ? v.e[q] : (T)0;
        } else {
#pragma unroll
            for (int q = 0; q < EPL; ++q) {
                const bool ok = row < M && kk + q < K;
                const T x = load_share<NT>(base + (ok ? (size_t)row * K + kk + q : 0));
                v.e[q] = ok ? x : (T)0;
            }
        }
        return v;
    };
    // lane -> LDS: written as (row RPL j + lane / LPR, k position lane % LPR), read back as
    // (row lane % 32, k 16 (lane / 32) ..)
    char *mine = turn[wave];
    auto turn_and_store = [&](const Pair (&v)[NL], char *dst) {
        __syncthreads();                                    // the previous round's reads are done
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            Pair d;
#pragma unroll
            for (int q = 0; q < EPL; ++q) d.e[q] = to_digits<T>(v[j].e[q]);
            *(Pair *)(mine + (RPL * j + lane / LPR) * kRowBytes + (lane % LPR) * 16) = d;
        }
        __syncthreads();
        T w[16];
#pragma unroll
        for (int j = 0; j < 16 / EPL; ++j) {
            Pair d = *(const Pair *)(mine + (lane % 32) * kRowBytes + (lane / 32) * (16 * ND) + j * 16);
#pragma unroll
            for (int q = 0; q < EPL; ++q) w[EPL * j + q] = d.e[q];
        }
        if (active) store_digit_rows<T, NT>(w, dst);
    };

    Pair opened[NL], first[KEEP ? NL : 1];
#pragma unroll
    for (int j = 0; j < NL; ++j)
#pragma unroll
        for (int q = 0; q < EPL; ++q) opened[j].e[q] = 0;
    // 16-byte rings keep the party loop rolled: unrolled, the loads of all parties are hoisted to the
    // top and the live values exceed the register file
    constexpr int kPartyUnroll = KEEP ? NP : 1;
#pragma unroll kPartyUnroll
    for (int i = 0; i < NP; ++i) {
        const T *v = a.val + (size_t)i * party_stride + (size_t)b * mat;
        const T *t = a.tri + (size_t)i * party_stride + (size_t)b * mat;
        Pair tv[NL];
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const int row = blk * 32 + RPL * j + lane / LPR;
            tv[j] = load(t, row);
            Pair xv = load(v, row);
#pragma unroll
            for (int q = 0; q < EPL; ++q) opened[j].e[q] += xv.e[q] - tv[j].e[q];
        }
        if (i == 0) {
            if constexpr (KEEP) {
#pragma unroll
                for (int j = 0; j < NL; ++j) first[j] = tv[j];
            }
        } else {
            turn_and_store(tv, frag(i + 1));
        }
    }
    turn_and_store(opened, frag(0));
    if constexpr (KEEP) {
        if (RIGHT) {
#pragma unroll
            for (int j = 0; j < NL; ++j)
#pragma unroll
                for (int q = 0; q < EPL; ++q) first[j].e[q] += opened[j].e[q];
        }
        turn_and_store(first, frag(1));
    } else {
        Pair tv[NL];
        const T *t = a.tri + (size_t)b * mat;
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            tv[j] = load(t, blk * 32 + RPL * j + lane / LPR);
            if (RIGHT) {
#pragma unroll
                for (int q = 0; q < EPL; ++q) tv[j].e[q] += opened[j].e[q];
            }
        }
        turn_and_store(tv, frag(1));
    }
}
template <int WAVES> __host__ __device__ inline unsigned pack_left_blocks(int nblk, int KT) { return (unsigned)(((long)nblk * KT + WAVES - 1) / WAVES); }

template <int NP, class T, bool VEC, int WAVES, bool RIGHT, bool NT>
__global__ __launch_bounds__(64 * WAVES) void pack_left_kernel(PackArgs<T> a)
{
    pack_left_body<NP, T, VEC, WAVES, RIGHT, NT>(a, blockIdx.x, blockIdx.z);
}

template <int NP, class T, bool VEC, int WAVES, bool RIGHT, bool NT>
__global__ __launch_bounds__(64 * WAVES) void pack_left_grouped_kernel(GroupTable<PackArgs<T>> t)
{
    const int gi = group_of(t, blockIdx.x);
    const PackArgs<T> a = t.e[gi];
    const unsigned local = blockIdx.x - t.first[gi], per_batch = pack_left_blocks<WAVES>(a.nblk, a.KT);
    pack_left_body<NP, T, VEC, WAVES, RIGHT, NT>(a, local % per_batch, (int)(local / per_batch));
}

// One direct-to-LDS load: 64 lanes x 16 bytes from src + lane*16 to the LDS address lds_dst + lane*16.
// Issued through inline assembly so that the compiler's LDS-DMA bookkeeping does not serialise the
// software pipeline; completion is awaited explicitly (wait_loads) before the workgroup barrier.
// The instruction takes its LDS base from m0, a register the compiler reserves for its own use and
// does not accept in a clobber list, so the statement puts back the value it found there (m0 is read
// when the load issues, so restoring it right after is safe).
__device__ inline void load_fragment_to_lds(const char *src, u32 lds_dst, u32 lane16)
{
    u32 saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0) : "v"(lane16), "s"(src), "s"(lds_dst) : "memory");
}
template <int N> __device__ inline void wait_loads() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }
__device__ inline void wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ inline void workgroup_barrier() { asm volatile("s_barrier" ::: "memory"); }

// Output tile of a workgroup.  Workgroup ids are dealt round-robin to the 8 XCDs; each XCD gets a
// contiguous range of the work items, so that workgroups sharing an L2 also share operand fragments,
// and walks the tiles of a matrix in 4-tile-tall column strips.
__device__ inline long xcd_contiguous_id(long id, long total)
{
    const long chunk = (total + 7) / 8;
    const long full = total - (chunk - 1) * 8;       // XCDs that own `chunk` items (the rest own chunk-1)
    const int xcd = (int)(id % 8);
    const long within = id / 8;
    return xcd < full ? xcd * chunk + within : full * chunk + (xcd - full) * (chunk - 1) + within;
}
struct TileId { int pb, tm, tn; };     // party * batch + b, tile row, tile column
__device__ inline TileId tile_of(long id, int tilesM, int tilesN)
{
    const int per_mat = tilesM * tilesN;
    TileId r;
    r.pb = (int)(id / per_mat);
    int t = (int)(id % per_mat);
    constexpr int GROUP = 4;
    const int strip = t / (GROUP * tilesN);
    const int strip_h = min(GROUP, tilesM - strip * GROUP);
    t -= strip * GROUP * tilesN;
    r.tm = strip * GROUP + t % strip_h;
    r.tn = t / strip_h;
    return r;
}
__device__ inline TileId map_tile(long id, int tilesM, int tilesN, long total)
{
    return tile_of(xcd_contiguous_id(id, total), tilesM, tilesN);
}

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Launches the pack kernels of one Beaver matmul: left operands from X, A; right operands from Y, B.
// Calls fn(std::true_type) when one side's share streams exceed the caches, fn(std::false_type) otherwise.
template <class T, class F> inline void for_pack_streaming(int n, int batch, int rows, int cols, F &&fn)
{
    if ((size_t)n * batch * rows * cols * sizeof(T) >= kPackStreamingBytes) fn(std::true_type());
    else fn(std::false_type());
}

template <class T>
inline void launch_pack_left(const MatmulArgsT<T> &a, char *packA, int nblkA, int KT, hipStream_t s)
{
    PackArgs<T> pa{a.X, a.A, packA, a.n, a.batch, a.M, a.K, nblkA, KT};
    constexpr int WAVES = sizeof(T) <= 8 ? 4 : 2;
    constexpr int EPL = 16 / sizeof(T);
    const bool vec = a.K % EPL == 0;                     // rows 16-byte aligned
    for_party_count(a.n, [&](auto np) {
        constexpr int NP = decltype(np)::value;
        for_pack_streaming<T>(a.n, a.batch, a.M, a.K, [&](auto nt) {
            constexpr bool NT = decltype(nt)::value;
            dim3 ga(pack_left_blocks<WAVES>(nblkA, KT), 1, a.batch);
            if (vec) pack_left_kernel<NP, T, true, WAVES, false, NT><<<ga, 64 * WAVES, 0, s>>>(pa);
            else pack_left_kernel<NP, T, false, WAVES, false, NT><<<ga, 64 * WAVES, 0, s>>>(pa);
        });
    });
}

template <class T>
inline void launch_pack_right(const MatmulArgsT<T> &a, char *packB, int nblkB, int KT, hipStream_t s)
{
    constexpr int WAVES = sizeof(T) <= 8 ? 4 : 2;
    constexpr int EPL = 16 / sizeof(T);
    const bool vec = a.K % EPL == 0;
    for_party_count(a.n, [&](auto np) {
        constexpr int NP = decltype(np)::value;
        for_pack_streaming<T>(a.n, a.batch, a.K, a.N, [&](auto nt) {
            constexpr bool NT = decltype(nt)::value;
            if (a.y_transposed) {                        // Y, B stored [N][K]: rows of the source are fragment rows
                PackArgs<T> pb{a.Y, a.B, packB, a.n, a.batch, a.N, a.K, nblkB, KT};
                dim3 gb(pack_left_blocks<WAVES>(nblkB, KT), 1, a.batch);
                if (vec) pack_left_kernel<NP, T, true, WAVES, true, NT><<<gb, 64 * WAVES, 0, s>>>(pb);
                else pack_left_kernel<NP, T, false, WAVES, true, NT><<<gb, 64 * WAVES, 0, s>>>(pb);
            } else {
                PackArgs<T> pb{a.Y, a.B, packB, a.n, a.batch, a.K, a.N, nblkB, KT};
                dim3 gb(pack_right_blocks(nblkB, KT), 1, a.batch);
                pack_right_kernel<NP, T, NT><<<gb, 256, 0, s>>>(pb);
            }
        });
    });
}

template <class T>
inline void launch_pack(const MatmulArgsT<T> &a, char *packA, char *packB, int nblkA, int nblkB, int KT, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_PACK, s);
    launch_pack_left<T>(a, packA, nblkA, KT, s);
    launch_pack_right<T>(a, packB, nblkB, KT, s);
}

}  // namespace
}  // namespace spin
