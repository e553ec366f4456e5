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
    if constexpr (NT && !std::is_same<V, u128>::value) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT, class V> __device__ inline void st(V *p, V v)
{
    if constexpr (NT && !std::is_same<V, u128>::value) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// V = u64x2 (two ring elements per lane) or u64 (odd counts, whose party rows
// are only 8-byte aligned).
template <class V> struct Lanes;
template <> struct Lanes<u64x2> { static constexpr int width = 2; };
template <> struct Lanes<u64>   { static constexpr int width = 1; };
template <> struct Lanes<u128>  { static constexpr int width = 1; };

template <class V> __device__ inline V gen(u64 key, u64 idx);
template <> __device__ inline u64 gen<u64>(u64 key, u64 idx) { return absorb(key, idx); }
template <> __device__ inline u64x2 gen<u64x2>(u64 key, u64 idx)
{
    u64x2 v; v.x = absorb(key, idx); v.y = absorb(key, idx + 1); return v;
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
template <int NP, class V, bool NT>
__global__ __launch_bounds__(kBlock) void share_kernel(const V *__restrict__ x, size_t nvec, PartyKeys keys,
                                                      V *__restrict__ shares)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= nvec) return;
    V rest = ld<NT>(x + v);
#pragma unroll
    for (int i = 1; i < NP; ++i) {
        V s = gen<V>(keys.key[i], v * Lanes<V>::width);
        st<NT>(shares + (size_t)i * nvec + v, s);
        rest -= s;
    }
    st<NT>(shares + v, rest);
}

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

// The combine of the signed probabilistic truncation (Section 4.4) on party shares y[] held in
// registers; steps as listed at spin_trunc in include/spin.h.
template <int NP, class T, bool NT>
__device__ inline void truncate_and_store(const T (&y)[NP], const T *__restrict__ r, const T *__restrict__ r_top,
                                          const T *__restrict__ r_msb, size_t count, size_t v, int f, T *out)
{
    constexpr int L = 8 * sizeof(T);               // ring width l
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
__global__ __launch_bounds__(kBlock) void trunc_kernel(const T *x, const T *__restrict__ r,
                                                      const T *__restrict__ r_top, const T *__restrict__ r_msb,
                                                      size_t count, int f, T *out)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= count) return;
    T y[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) y[i] = ld<NT>(x + (size_t)i * count + v);
    truncate_and_store<NP, T, NT>(y, r, r_top, r_msb, count, v, f, out);
}

// y_i = sum_j coef_j in_j,i (+ constant for party 0), then the truncation above when TRUNC
// (Section 4.3 Addition/Scaling; Section 4.4 Polynomial evaluation: one deferred truncation).
// The term loop is a run-time loop; every iteration issues one load per party.
template <int NP, bool TRUNC, bool NT>
__global__ __launch_bounds__(kBlock) void lincomb_trunc_kernel(LincombTerms t, u64 constant, const u64 *__restrict__ r,
                                                              const u64 *__restrict__ r_top,
                                                              const u64 *__restrict__ r_msb, size_t count, int f,
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

template <int NP, bool MASK>
__global__ __launch_bounds__(kBlock) void bopen_kernel(const u64 *__restrict__ shares, const u64 *__restrict__ mask,
                                                      size_t count, u64 *__restrict__ out)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= count) return;
    u64 s[NP], m[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        s[i] = shares[(size_t)i * count + v];
        if (MASK) m[i] = mask[(size_t)i * count + v];
    }
    u64 acc = 0;
#pragma unroll
    for (int i = 0; i < NP; ++i) acc ^= MASK ? s[i] ^ m[i] : s[i];
    out[v] = acc;
}

template <int NP>
__global__ __launch_bounds__(kBlock) void beaver_and_kernel(const u64 *x, const u64 *y, const u64 *a, const u64 *b,
                                                           const u64 *c, size_t count, u64 *z)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= count) return;
    u64 xv[NP], yv[NP], av[NP], bv[NP], cv[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        size_t o = (size_t)i * count + v;
        xv[i] = x[o]; yv[i] = y[o]; av[i] = a[o]; bv[i] = b[o]; cv[i] = c[o];
    }
    u64 e = 0, f = 0;
#pragma unroll
    for (int i = 0; i < NP; ++i) { e ^= xv[i] ^ av[i]; f ^= yv[i] ^ bv[i]; }
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        u64 bi = bv[i];
        if (i == 0) bi ^= f;                       // (e & b_0) ^ (e & f) = e & (b_0 ^ f)
        z[(size_t)i * count + v] = cv[i] ^ (e & bi) ^ (av[i] & f);
    }
}

inline unsigned grid_for(size_t n) { return (unsigned)((n + kBlock - 1) / kBlock); }

// Calls fn(std::true_type) for calls that stream more than the caches hold, fn(std::false_type) otherwise.
template <class F> inline void for_streaming(size_t bytes, F &&fn)
{
    if (bytes >= kStreamingBytes) fn(std::true_type());
    else fn(std::false_type());
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
            share_kernel<NP, u64x2, false><<<grid_for(count / 2), kBlock, 0, s>>>((const u64x2 *)x, count / 2, keys,
                                                                                 (u64x2 *)shares);
        else
            share_kernel<NP, u64, false><<<grid_for(count), kBlock, 0, s>>>(x, count, keys, shares);
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
            if (mask) open_kernel<NP, true, T, NT><<<grid_for(count), kBlock, 0, s>>>(shares, mask, count, out);
            else open_kernel<NP, false, T, NT><<<grid_for(count), kBlock, 0, s>>>(shares, nullptr, count, out);
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
            beaver_mul_kernel<decltype(np)::value, T, decltype(nt)::value><<<grid_for(count), kBlock, 0, s>>>(
                x, y, a, b, c, count, z);
        });
    });
    return check_launch("spin_beaver_mul");
}

template <class T>
spin_status launch_trunc(int n, size_t count, int f, const T *x, const T *r, const T *r_top, const T *r_msb, T *out,
                         hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_TRUNC, s);
    for_party_count(n, [&](auto np) {
        for_streaming((size_t)n * count * sizeof(T), [&](auto nt) {
            trunc_kernel<decltype(np)::value, T, decltype(nt)::value><<<grid_for(count), kBlock, 0, s>>>(
                x, r, r_top, r_msb, count, f, out);
        });
    });
    return check_launch("spin_trunc");
}

spin_status launch_share128(const u128 *x, size_t count, int n, const PartyKeys &keys, u128 *shares, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_SHARE, s);
    for_party_count(n, [&](auto np) {
        share_kernel<decltype(np)::value, u128, false><<<grid_for(count), kBlock, 0, s>>>(x, count, keys, shares);
    });
    return check_launch("spin128_share");
}

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
        if (mask) bopen_kernel<NP, true><<<grid_for(count), kBlock, 0, s>>>(shares, mask, count, out);
        else bopen_kernel<NP, false><<<grid_for(count), kBlock, 0, s>>>(shares, nullptr, count, out);
    });
    return check_launch("spin_bopen");
}

spin_status launch_beaver_and(int n, size_t count, const u64 *x, const u64 *y, const u64 *a, const u64 *b,
                              const u64 *c, u64 *z, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_BINARY, s);
    for_party_count(n, [&](auto np) {
        beaver_and_kernel<decltype(np)::value><<<grid_for(count), kBlock, 0, s>>>(x, y, a, b, c, count, z);
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
