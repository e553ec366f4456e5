// Elementwise share kernels: generator fill, sharing, opening, the fused
// Beaver update for arrays, truncation, and the public-coefficient linear
// combination with fused truncation.  All of them are pure HBM streams: one
// pass, every party's operand read exactly once, opened values (e, f, c) kept
// in registers because all parties are resident on the same GPU.
//
// Lane width.  The write-dominated kernels (random, share) move 16 bytes per
// lane.  The kernels that read many party-major streams at once (open,
// beaver_mul, trunc, lincomb: up to 6n concurrent streams) move 8 bytes per
// lane: measured on MI355X at n = 5 and 2^24 elements, 8-byte lanes sustain
// about 8 % more HBM bandwidth than 16-byte lanes for that access pattern
// (5.6 against 5.2 TB/s for trunc).
#include <initializer_list>

#include "common.hpp"

namespace spin {
namespace {

constexpr int kBlock = 256;

// Streaming accesses.  Tensors far larger than the caches are read and written exactly once, and
// non-temporal loads and stores (no cache retention) measured 14 % faster on the 25-stream truncation
// pattern (n = 5, 2^24 elements, same process: 6.4 against 5.6 TB/s).
// Small tensors keep ordinary accesses so that the next kernel finds them in L2 / Infinity Cache.
constexpr size_t kStreamingBytes = (size_t)64 << 20;    // per call, all parties together
template <bool NT, class V> __device__ inline V ld(const V *p)
{
    if constexpr (NT && std::is_same<V, u128>::value) {          // the builtin takes no __int128: same 16 bytes as u64x2
        const u64x2 w = __builtin_nontemporal_load((const u64x2 *)p);
        return (u128)w.x | ((u128)w.y << 64);
    } else if constexpr (NT) {
        return __builtin_nontemporal_load(p);
    } else {
        return *p;
    }
}
template <bool NT, class V> __device__ inline void st(V *p, V v)
{
    if constexpr (NT && std::is_same<V, u128>::value) {
        u64x2 w; w.x = (u64)v; w.y = (u64)(v >> 64);
        __builtin_nontemporal_store(w, (u64x2 *)p);
    } else if constexpr (NT) {
        __builtin_nontemporal_store(v, p);
    } else {
        *p = v;
    }
}

// Lane types.  V = u64x2 (two ring elements per lane) or u64 (odd counts, whose party rows are only
// 8-byte aligned); for the 4-byte ring u32x4 / u32x2 / u32 likewise.  `bits` is the ring width l.
template <class V> struct Lanes;
template <> struct Lanes<u64x2> { static constexpr int width = 2; };
template <> struct Lanes<u64>   { static constexpr int width = 1, bits = 64; };
template <> struct Lanes<u128>  { static constexpr int width = 1, bits = 128; };
template <> struct Lanes<u32x4> { static constexpr int width = 4; };
template <> struct Lanes<u32x2> { static constexpr int width = 2, bits = 32; };
template <> struct Lanes<u32>   { static constexpr int width = 1, bits = 32; };

template <class V> __device__ inline V gen(u64 key, u64 idx);
template <> __device__ inline u64 gen<u64>(u64 key, u64 idx) { return absorb(key, idx); }
template <> __device__ inline u64x2 gen<u64x2>(u64 key, u64 idx)
{
    u64x2 v; v.x = absorb(key, idx); v.y = absorb(key, idx + 1); return v;
}

// a 32-bit generator word is the low half of the 64-bit output at the same index
template <> __device__ inline u32 gen<u32>(u64 key, u64 idx) { return (u32)absorb(key, idx); }
template <> __device__ inline u32x2 gen<u32x2>(u64 key, u64 idx)
{
    u32x2 v; v.x = (u32)absorb(key, idx); v.y = (u32)absorb(key, idx + 1); return v;
}
template <> __device__ inline u32x4 gen<u32x4>(u64 key, u64 idx)
{
    u32x4 v;
    v.x = (u32)absorb(key, idx); v.y = (u32)absorb(key, idx + 1);
    v.z = (u32)absorb(key, idx + 2); v.w = (u32)absorb(key, idx + 3);
    return v;
}

// a 128-bit generator word is the pair of 64-bit outputs 2 idx (low) and 2 idx + 1 (high)
template <> __device__ inline u128 gen<u128>(u64 key, u64 idx)
{
    return (u128)absorb(key, 2 * idx) | ((u128)absorb(key, 2 * idx + 1) << 64);
}

template <class V>
__global__ __launch_bounds__(kBlock) void random_kernel(V *__restrict__ out, size_t nvec, u64 key, u64 first_idx)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= nvec) return;
    out[v] = gen<V>(key, first_idx + v * Lanes<V>::width);
}

// shares[i] = generator output for i >= 1, shares[0] = x - sum of the others (Section 4.1).
// A thread handles kShareU lane vectors a block apart: two independent generator chains per party and
// twice the stores in flight (measured 0.74 -> 0.76 of HBM peak at 5 parties x 2^24; four is slower again).
constexpr int kShareU = 2;
template <int NP, class V, bool NT>
__global__ __launch_bounds__(kBlock) void share_kernel(const V *__restrict__ x, size_t nvec, PartyKeys keys,
                                                      V *__restrict__ shares)
{
    const size_t v0 = (size_t)blockIdx.x * (kBlock * kShareU) + threadIdx.x;
    V rest[kShareU];
#pragma unroll
    for (int u = 0; u < kShareU; ++u) {
        const size_t v = v0 + (size_t)u * kBlock;
        rest[u] = v < nvec ? ld<NT>(x + v) : V{};
    }
#pragma unroll
    for (int i = 1; i < NP; ++i) {
#pragma unroll
        for (int u = 0; u < kShareU; ++u) {
            const size_t v = v0 + (size_t)u * kBlock;
            V s = gen<V>(keys.key[i], v * Lanes<V>::width);
            if (v < nvec) st<NT>(shares + (size_t)i * nvec + v, s);
            rest[u] -= s;
        }
    }
#pragma unroll
    for (int u = 0; u < kShareU; ++u) {
        const size_t v = v0 + (size_t)u * kBlock;
        if (v < nvec) st<NT>(shares + v, rest[u]);
    }
}
inline unsigned share_grid(size_t nvec) { return (unsigned)((nvec + (size_t)kBlock * kShareU - 1) / ((size_t)kBlock * kShareU)); }

// out = sum_i (shares_i - mask_i): the party-axis reduction that replaces the network exchange.
template <int NP, bool MASK, class T, bool NT>
__global__ __launch_bounds__(kBlock) void open_kernel(const T *__restrict__ shares, const T *__restrict__ mask,
                                                     size_t count, T *__restrict__ out)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= count) return;
    T s[NP], m[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        s[i] = ld<NT>(shares + (size_t)i * count + v);
        if (MASK) m[i] = ld<NT>(mask + (size_t)i * count + v);
    }
    T acc = 0;
#pragma unroll
    for (int i = 0; i < NP; ++i) acc += MASK ? s[i] - m[i] : s[i];
    st<NT>(out + v, acc);
}

// z_i = c_i + e*b_i + a_i*f (+ e*f for party 0) with e, f opened in registers (Section 4.3).
// z may alias an input: a thread reads all of its inputs before it writes.
template <int NP, class T, bool NT>
__global__ __launch_bounds__(kBlock) void beaver_mul_kernel(const T *x, const T *y, const T *a, const T *b,
                                                           const T *c, size_t count, T *z)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= count) return;
    T xv[NP], yv[NP], av[NP], bv[NP], cv[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        size_t o = (size_t)i * count + v;
        xv[i] = ld<NT>(x + o); yv[i] = ld<NT>(y + o); av[i] = ld<NT>(a + o); bv[i] = ld<NT>(b + o);
        cv[i] = ld<NT>(c + o);
    }
    T e = 0, f = 0;
#pragma unroll
    for (int i = 0; i < NP; ++i) { e += xv[i] - av[i]; f += yv[i] - bv[i]; }
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        T bi = bv[i];
        if (i == 0) bi += f;                       // folds the public e*f into party 0's term
        st<NT>(z + (size_t)i * count + v, cv[i] + e * bi + av[i] * f);
    }
}

// The same update with one factor tiled (Section 7.3: E * R with R repeated along an axis): x and a hold
// one element per (outer, mid) row (OVER_INNER) or per (outer, inner) column of the [outer][mid][inner]
// tensors y, b, c, z.  The tiled array is never materialised: every thread reads its factor's 2n words
// from the small arrays (cache hits after the first touch) and streams 4n words of the large ones.
template <int NP, bool OVER_INNER, bool NT>
__global__ __launch_bounds__(kBlock) void beaver_mul_bcast_kernel(const u64 *__restrict__ x, const u64 *y,
                                                                 const u64 *__restrict__ a, const u64 *b,
                                                                 const u64 *c, size_t small_count, size_t count,
                                                                 size_t mid, size_t inner, u64 *z)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= count) return;
    const size_t sidx = OVER_INNER ? v / inner : v / (mid * inner) * inner + v % inner;
    u64 xv[NP], yv[NP], av[NP], bv[NP], cv[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        size_t o = (size_t)i * count + v, so = (size_t)i * small_count + sidx;
        xv[i] = x[so]; av[i] = a[so];
        yv[i] = ld<NT>(y + o); bv[i] = ld<NT>(b + o); cv[i] = ld<NT>(c + o);
    }
    u64 e = 0, f = 0;
#pragma unroll
    for (int i = 0; i < NP; ++i) { e += xv[i] - av[i]; f += yv[i] - bv[i]; }
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        u64 bi = bv[i];
        if (i == 0) bi += f;
        st<NT>(z + (size_t)i * count + v, cv[i] + e * bi + av[i] * f);
    }
}

// The combine of the signed probabilistic truncation (Section 4.4) on party shares y[] held in
// registers; steps as listed at spin_trunc in include/spin.h.  Every tuple word is read before the first
// store, and no pointer is declared restrict, so `out` may be any of the inputs.
template <int NP, class T, bool NT>
__device__ inline void truncate_and_store(const T (&y)[NP], const T *r, const T *r_top, const T *r_msb, size_t count,
                                          size_t v, int f, T *out)
{
    constexpr int L = Lanes<T>::bits;              // ring width l
    T rt[NP], rm[NP];
    T c = (T)1 << (L - 2);
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        size_t o = (size_t)i * count + v;
        rt[i] = ld<NT>(r_top + o); rm[i] = ld<NT>(r_msb + o);
        c += y[i] + ld<NT>(r + o);
    }
    const T topmask = (((T)1 << (L - 1 - f)) - 1);
    const T c_msb = c >> (L - 1);
    const T c_top = (c >> f) & topmask;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        T b = rm[i] - 2 * c_msb * rm[i];
        T o = (b << (L - 1 - f)) - rt[i];
        if (i == 0) o += (c_msb << (L - 1 - f)) + c_top - ((T)1 << (L - 2 - f));
        st<NT>(out + (size_t)i * count + v, o);
    }
}

template <int NP, class T, bool NT>
__global__ __launch_bounds__(kBlock) void trunc_kernel(const T *x, const T *r, const T *r_top, const T *r_msb,
                                                      size_t count, int f, T *out)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= count) return;
    T y[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) y[i] = ld<NT>(x + (size_t)i * count + v);
    truncate_and_store<NP, T, NT>(y, r, r_top, r_msb, count, v, f, out);
}

// Fixed-point multiplication in one pass: the Beaver update of beaver_mul_kernel, then the truncation of the
// doubled precision (Section 4.3: a product carries precision 2p; Section 4.4 brings it back).  The
// product shares stay in registers, so they are neither written nor read back: 9n words per element
// instead of 6n + 5n.
template <int NP, bool NT>
__global__ __launch_bounds__(kBlock) void beaver_mul_trunc_kernel(const u64 *x, const u64 *y, const u64 *a,
                                                                 const u64 *b, const u64 *c, const u64 *r,
                                                                 const u64 *r_top, const u64 *r_msb, size_t count,
                                                                 int f, u64 *out)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= count) return;
    u64 xv[NP], yv[NP], av[NP], bv[NP], z[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        size_t o = (size_t)i * count + v;
        xv[i] = ld<NT>(x + o); yv[i] = ld<NT>(y + o); av[i] = ld<NT>(a + o); bv[i] = ld<NT>(b + o);
        z[i] = ld<NT>(c + o);
    }
    u64 e = 0, g = 0;
#pragma unroll
    for (int i = 0; i < NP; ++i) { e += xv[i] - av[i]; g += yv[i] - bv[i]; }
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        u64 bi = bv[i];
        if (i == 0) bi += g;
        z[i] += e * bi + av[i] * g;
    }
    truncate_and_store<NP, u64, NT>(z, r, r_top, r_msb, count, v, f, out);
}

// y_i = sum_j coef_j in_j,i (+ constant for party 0), then the truncation above when TRUNC
// (Section 4.3 Addition/Scaling; Section 4.4 Polynomial evaluation: one deferred truncation).
// The term loop is a run-time loop; every iteration issues one load per party.
template <int NP, bool TRUNC, bool NT>
__global__ __launch_bounds__(kBlock) void lincomb_trunc_kernel(LincombTerms t, u64 constant, const u64 *r,
                                                              const u64 *r_top, const u64 *r_msb, size_t count, int f,
                                                              u64 *out)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= count) return;
    u64 y[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) y[i] = i == 0 ? constant : 0;
    for (int j = 0; j < t.terms; ++j) {
        const u64 *src = t.in[j];
        const u64 cf = t.coef[j];
#pragma unroll
        for (int i = 0; i < NP; ++i) y[i] += cf * ld<NT>(src + (size_t)i * count + v);
    }
    if (TRUNC) {
        truncate_and_store<NP, u64, NT>(y, r, r_top, r_msb, count, v, f, out);
    } else {
#pragma unroll
        for (int i = 0; i < NP; ++i) st<NT>(out + (size_t)i * count + v, y[i]);
    }
}

// Fixed64 -> Fixed32 (Section 7.1): every party keeps the low 32 bits of its own share; the sum of the
// low halves is the value mod 2^32, which is the value itself while it fits 32 bits.
template <class VI, class VO, bool NT>
__global__ __launch_bounds__(kBlock) void cast_low_kernel(const VI *__restrict__ in, size_t nvec, VO *__restrict__ out)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= nvec) return;
    st<NT>(out + v, __builtin_convertvector(ld<NT>(in + v), VO));
}
template <bool NT>
__global__ __launch_bounds__(kBlock) void cast_low_kernel1(const u64 *__restrict__ in, size_t count, u32 *__restrict__ out)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= count) return;
    st<NT>(out + v, (u32)ld<NT>(in + v));
}

// ---- binary sharing: the same three streams with XOR for + and AND for * (Section 4.1, 4.3) ----
template <int NP>
__global__ __launch_bounds__(kBlock) void bshare_kernel(const u64 *__restrict__ x, size_t count, PartyKeys keys,
                                                       u64 *__restrict__ shares)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= count) return;
    u64 rest = x[v];
#pragma unroll
    for (int i = 1; i < NP; ++i) {
        u64 s = absorb(keys.key[i], v);
        shares[(size_t)i * count + v] = s;
        rest ^= s;
    }
    shares[v] = rest;
}

template <int NP, bool MASK, bool NT>
__global__ __launch_bounds__(kBlock) void bopen_kernel(const u64 *__restrict__ shares, const u64 *__restrict__ mask,
                                                      size_t count, u64 *__restrict__ out)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= count) return;
    u64 s[NP], m[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        s[i] = ld<NT>(shares + (size_t)i * count + v);
        if (MASK) m[i] = ld<NT>(mask + (size_t)i * count + v);
    }
    u64 acc = 0;
#pragma unroll
    for (int i = 0; i < NP; ++i) acc ^= MASK ? s[i] ^ m[i] : s[i];
    st<NT>(out + v, acc);
}

template <int NP, bool NT>
__global__ __launch_bounds__(kBlock) void beaver_and_kernel(const u64 *x, const u64 *y, const u64 *a, const u64 *b,
                                                           const u64 *c, size_t count, u64 *z)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= count) return;
    u64 xv[NP], yv[NP], av[NP], bv[NP], cv[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        size_t o = (size_t)i * count + v;
        xv[i] = ld<NT>(x + o); yv[i] = ld<NT>(y + o); av[i] = ld<NT>(a + o); bv[i] = ld<NT>(b + o);
        cv[i] = ld<NT>(c + o);
    }
    u64 e = 0, f = 0;
#pragma unroll
    for (int i = 0; i < NP; ++i) { e ^= xv[i] ^ av[i]; f ^= yv[i] ^ bv[i]; }
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        u64 bi = bv[i];
        if (i == 0) bi ^= f;                       // (e & b_0) ^ (e & f) = e & (b_0 ^ f)
        st<NT>(z + (size_t)i * count + v, cv[i] ^ (e & bi) ^ (av[i] & f));
    }
}

inline unsigned grid_for(size_t n) { return (unsigned)((n + kBlock - 1) / kBlock); }

// Calls fn(std::true_type) for calls that stream more than the caches hold, fn(std::false_type) otherwise.
template <class F> inline void for_streaming(size_t bytes, F &&fn)
{
    if (bytes >= kStreamingBytes) fn(std::true_type());
    else fn(std::false_type());
}

// Calls fn(lane type tag, number of lane vectors).  The 4-byte ring moves two elements per lane when
// the count is even (party rows then stay 8-byte aligned) and every pointer is 8-byte aligned; other
// rings move one element per lane.
template <class T, class F> inline void for_lane_type(size_t count, std::initializer_list<const void *> ptrs, F &&fn)
{
    if constexpr (std::is_same<T, u32>::value) {
        bool pair = count % 2 == 0;
        for (const void *p : ptrs) pair = pair && ((uintptr_t)p % 8 == 0);
        if (pair) { fn((u32x2 *)nullptr, count / 2); return; }
    }
    fn((T *)nullptr, count);
}

}  // namespace

spin_status launch_random(u64 *out, size_t count, u64 key, u64 first_idx, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_RANDOM, s);
    if (count % 2 == 0)
        random_kernel<u64x2><<<grid_for(count / 2), kBlock, 0, s>>>((u64x2 *)out, count / 2, key, first_idx);
    else
        random_kernel<u64><<<grid_for(count), kBlock, 0, s>>>(out, count, key, first_idx);
    return check_launch("spin_random");
}

spin_status launch_share(const u64 *x, size_t count, int n, const PartyKeys &keys, u64 *shares, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_SHARE, s);
    for_party_count(n, [&](auto np) {
        constexpr int NP = decltype(np)::value;
        // ordinary stores: in a pipeline the shares are read again at once (by the pack kernels), and
        // non-temporal stores, although faster in isolation, measured slower there
        if (count % 2 == 0)
            share_kernel<NP, u64x2, false><<<share_grid(count / 2), kBlock, 0, s>>>((const u64x2 *)x, count / 2, keys,
                                                                                 (u64x2 *)shares);
        else
            share_kernel<NP, u64, false><<<share_grid(count), kBlock, 0, s>>>(x, count, keys, shares);
    });
    return check_launch("spin_share");
}

template <class T>
spin_status launch_open(const T *shares, const T *mask, size_t count, int n, T *out, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_OPEN, s);
    for_party_count(n, [&](auto np) {
        constexpr int NP = decltype(np)::value;
        for_streaming((size_t)n * count * sizeof(T), [&](auto nt) {
            constexpr bool NT = decltype(nt)::value;
            for_lane_type<T>(count, {shares, mask, out}, [&](auto *tag, size_t nvec) {
                using V = std::remove_pointer_t<decltype(tag)>;
                if (mask)
                    open_kernel<NP, true, V, NT><<<grid_for(nvec), kBlock, 0, s>>>((const V *)shares, (const V *)mask,
                                                                                  nvec, (V *)out);
                else
                    open_kernel<NP, false, V, NT><<<grid_for(nvec), kBlock, 0, s>>>((const V *)shares, nullptr, nvec,
                                                                                   (V *)out);
            });
        });
    });
    return check_launch("spin_open");
}

template <class T>
spin_status launch_beaver_mul(int n, size_t count, const T *x, const T *y, const T *a, const T *b, const T *c, T *z,
                              hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_BEAVER_MUL, s);
    for_party_count(n, [&](auto np) {
        for_streaming((size_t)n * count * sizeof(T), [&](auto nt) {
            for_lane_type<T>(count, {x, y, a, b, c, z}, [&](auto *tag, size_t nvec) {
                using V = std::remove_pointer_t<decltype(tag)>;
                beaver_mul_kernel<decltype(np)::value, V, decltype(nt)::value><<<grid_for(nvec), kBlock, 0, s>>>(
                    (const V *)x, (const V *)y, (const V *)a, (const V *)b, (const V *)c, nvec, (V *)z);
            });
        });
    });
    return check_launch("spin_beaver_mul");
}

spin_status launch_beaver_mul_trunc(int n, size_t count, int f, const u64 *x, const u64 *y, const u64 *a, const u64 *b,
                                    const u64 *c, const u64 *r, const u64 *r_top, const u64 *r_msb, u64 *out,
                                    hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_MUL_TRUNC, s);
    for_party_count(n, [&](auto np) {
        for_streaming((size_t)n * count * sizeof(u64), [&](auto nt) {
            beaver_mul_trunc_kernel<decltype(np)::value, decltype(nt)::value><<<grid_for(count), kBlock, 0, s>>>(
                x, y, a, b, c, r, r_top, r_msb, count, f, out);
        });
    });
    return check_launch("spin_beaver_mul_trunc");
}

spin_status launch_beaver_mul_bcast(int n, size_t outer, size_t mid, size_t inner, bool over_inner, const u64 *x,
                                    const u64 *y, const u64 *a, const u64 *b, const u64 *c, u64 *z, hipStream_t s)
{
    const size_t count = outer * mid * inner, small_count = outer * (over_inner ? mid : inner);
    if (small_count == count) return launch_beaver_mul<u64>(n, count, x, y, a, b, c, z, s);   // nothing is repeated
    KernelTimer timer(SPIN_KERNEL_BEAVER_MUL, s);
    for_party_count(n, [&](auto np) {
        constexpr int NP = decltype(np)::value;
        for_streaming((size_t)n * count * sizeof(u64), [&](auto nt) {
            constexpr bool NT = decltype(nt)::value;
            if (over_inner)
                beaver_mul_bcast_kernel<NP, true, NT><<<grid_for(count), kBlock, 0, s>>>(x, y, a, b, c, small_count,
                                                                                        count, mid, inner, z);
            else
                beaver_mul_bcast_kernel<NP, false, NT><<<grid_for(count), kBlock, 0, s>>>(x, y, a, b, c, small_count,
                                                                                         count, mid, inner, z);
        });
    });
    return check_launch("spin_beaver_mul_bcast");
}

template <class T>
spin_status launch_trunc(int n, size_t count, int f, const T *x, const T *r, const T *r_top, const T *r_msb, T *out,
                         hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_TRUNC, s);
    for_party_count(n, [&](auto np) {
        for_streaming((size_t)n * count * sizeof(T), [&](auto nt) {
            for_lane_type<T>(count, {x, r, r_top, r_msb, out}, [&](auto *tag, size_t nvec) {
                using V = std::remove_pointer_t<decltype(tag)>;
                trunc_kernel<decltype(np)::value, V, decltype(nt)::value><<<grid_for(nvec), kBlock, 0, s>>>(
                    (const V *)x, (const V *)r, (const V *)r_top, (const V *)r_msb, nvec, f, (V *)out);
            });
        });
    });
    return check_launch("spin_trunc");
}

spin_status launch_share128(const u128 *x, size_t count, int n, const PartyKeys &keys, u128 *shares, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_SHARE, s);
    for_party_count(n, [&](auto np) {
        share_kernel<decltype(np)::value, u128, false><<<share_grid(count), kBlock, 0, s>>>(x, count, keys, shares);
    });
    return check_launch("spin128_share");
}

spin_status launch_share32(const u32 *x, size_t count, int n, const PartyKeys &keys, u32 *shares, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_SHARE, s);
    for_party_count(n, [&](auto np) {
        constexpr int NP = decltype(np)::value;
        if (count % 4 == 0)
            share_kernel<NP, u32x4, false><<<share_grid(count / 4), kBlock, 0, s>>>((const u32x4 *)x, count / 4, keys,
                                                                                 (u32x4 *)shares);
        else if (count % 2 == 0)
            share_kernel<NP, u32x2, false><<<share_grid(count / 2), kBlock, 0, s>>>((const u32x2 *)x, count / 2, keys,
                                                                                 (u32x2 *)shares);
        else
            share_kernel<NP, u32, false><<<share_grid(count), kBlock, 0, s>>>(x, count, keys, shares);
    });
    return check_launch("spin32_share");
}

spin_status launch_cast_low(const u64 *in, size_t count, u32 *out, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_CAST, s);
    for_streaming(count * sizeof(u64), [&](auto nt) {
        constexpr bool NT = decltype(nt)::value;
        if (count % 2 == 0)
            cast_low_kernel<u64x2, u32x2, NT><<<grid_for(count / 2), kBlock, 0, s>>>((const u64x2 *)in, count / 2,
                                                                                    (u32x2 *)out);
        else
            cast_low_kernel1<NT><<<grid_for(count), kBlock, 0, s>>>(in, count, out);
    });
    return check_launch("spin_cast_64_to_32");
}

template spin_status launch_open<u32>(const u32 *, const u32 *, size_t, int, u32 *, hipStream_t);
template spin_status launch_beaver_mul<u32>(int, size_t, const u32 *, const u32 *, const u32 *, const u32 *, const u32 *,
                                            u32 *, hipStream_t);
template spin_status launch_trunc<u32>(int, size_t, int, const u32 *, const u32 *, const u32 *, const u32 *, u32 *,
                                       hipStream_t);
template spin_status launch_open<u64>(const u64 *, const u64 *, size_t, int, u64 *, hipStream_t);
template spin_status launch_open<u128>(const u128 *, const u128 *, size_t, int, u128 *, hipStream_t);
template spin_status launch_beaver_mul<u64>(int, size_t, const u64 *, const u64 *, const u64 *, const u64 *, const u64 *,
                                            u64 *, hipStream_t);
template spin_status launch_beaver_mul<u128>(int, size_t, const u128 *, const u128 *, const u128 *, const u128 *,
                                             const u128 *, u128 *, hipStream_t);
template spin_status launch_trunc<u64>(int, size_t, int, const u64 *, const u64 *, const u64 *, const u64 *, u64 *,
                                       hipStream_t);
template spin_status launch_trunc<u128>(int, size_t, int, const u128 *, const u128 *, const u128 *, const u128 *,
                                        u128 *, hipStream_t);

spin_status launch_bshare(const u64 *x, size_t count, int n, const PartyKeys &keys, u64 *shares, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_BINARY, s);
    for_party_count(n, [&](auto np) {
        bshare_kernel<decltype(np)::value><<<grid_for(count), kBlock, 0, s>>>(x, count, keys, shares);
    });
    return check_launch("spin_bshare");
}

spin_status launch_bopen(const u64 *shares, const u64 *mask, size_t count, int n, u64 *out, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_BINARY, s);
    for_party_count(n, [&](auto np) {
        constexpr int NP = decltype(np)::value;
        for_streaming((size_t)n * count * sizeof(u64), [&](auto nt) {
            constexpr bool NT = decltype(nt)::value;
            if (mask) bopen_kernel<NP, true, NT><<<grid_for(count), kBlock, 0, s>>>(shares, mask, count, out);
            else bopen_kernel<NP, false, NT><<<grid_for(count), kBlock, 0, s>>>(shares, nullptr, count, out);
        });
    });
    return check_launch("spin_bopen");
}

spin_status launch_beaver_and(int n, size_t count, const u64 *x, const u64 *y, const u64 *a, const u64 *b,
                              const u64 *c, u64 *z, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_BINARY, s);
    for_party_count(n, [&](auto np) {
        for_streaming((size_t)n * count * sizeof(u64), [&](auto nt) {
            beaver_and_kernel<decltype(np)::value, decltype(nt)::value><<<grid_for(count), kBlock, 0, s>>>(
                x, y, a, b, c, count, z);
        });
    });
    return check_launch("spin_beaver_and");
}

spin_status launch_lincomb_trunc(int n, size_t count, const LincombTerms &t, u64 constant, int f, const u64 *r,
                                 const u64 *r_top, const u64 *r_msb, u64 *out, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_LINCOMB, s);
    for_party_count(n, [&](auto np) {
        constexpr int NP = decltype(np)::value;
        for_streaming((size_t)n * count * sizeof(u64), [&](auto nt) {
            constexpr bool NT = decltype(nt)::value;
            if (f > 0)
                lincomb_trunc_kernel<NP, true, NT><<<grid_for(count), kBlock, 0, s>>>(t, constant, r, r_top, r_msb,
                                                                                     count, f, out);
            else
                lincomb_trunc_kernel<NP, false, NT><<<grid_for(count), kBlock, 0, s>>>(t, constant, nullptr, nullptr,
                                                                                      nullptr, count, 0, out);
        });
    });
    return check_launch("spin_lincomb_trunc");
}

}  // namespace spin
