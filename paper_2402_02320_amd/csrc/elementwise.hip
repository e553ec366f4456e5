// Elementwise share kernels: generator fill, sharing, opening, the fused
// Beaver update for arrays, and truncation.  All of them are pure HBM
// streams: one pass, every party's operand read exactly once, opened values
// (e, f, c) kept in registers because all parties are resident on the same GPU.
//
// Lane width.  The write-dominated kernels (random, share) move 16 bytes per
// lane.  The kernels that read many party-major streams at once (open,
// beaver_mul, trunc: up to 5n+n concurrent streams) move 8 bytes per lane:
// measured on MI355X at n = 5, 2^24 elements, 8-byte lanes sustain about 8 %
// more HBM bandwidth than 16-byte lanes for that access pattern.
#include "common.hpp"

namespace spin {
namespace {

constexpr int kBlock = 256;
constexpr bool kWideLanes = false;   // 16-byte lanes for the many-stream kernels (kept for measurement)

// V = u64x2 (two ring elements per lane) or u64 (odd counts, whose party rows
// are only 8-byte aligned).
template <class V> struct Lanes;
template <> struct Lanes<u64x2> { static constexpr int width = 2; };
template <> struct Lanes<u64>   { static constexpr int width = 1; };

template <class V> __device__ inline V gen(u64 key, u64 idx);
template <> __device__ inline u64 gen<u64>(u64 key, u64 idx) { return absorb(key, idx); }
template <> __device__ inline u64x2 gen<u64x2>(u64 key, u64 idx)
{
    u64x2 v; v.x = absorb(key, idx); v.y = absorb(key, idx + 1); return v;
}

template <class V>
__global__ __launch_bounds__(kBlock) void random_kernel(V *__restrict__ out, size_t nvec, u64 key, u64 first_idx)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= nvec) return;
    out[v] = gen<V>(key, first_idx + v * Lanes<V>::width);
}

// shares[i] = generator output for i >= 1, shares[0] = x - sum of the others (Section 4.1).
template <int NP, class V>
__global__ __launch_bounds__(kBlock) void share_kernel(const V *__restrict__ x, size_t nvec, PartyKeys keys,
                                                      V *__restrict__ shares)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= nvec) return;
    V rest = x[v];
#pragma unroll
    for (int i = 1; i < NP; ++i) {
        V s = gen<V>(keys.key[i], v * Lanes<V>::width);
        shares[(size_t)i * nvec + v] = s;
        rest -= s;
    }
    shares[v] = rest;
}

// out = sum_i (shares_i - mask_i): the party-axis reduction that replaces the network exchange.
template <int NP, bool MASK, class V>
__global__ __launch_bounds__(kBlock) void open_kernel(const V *__restrict__ shares, const V *__restrict__ mask,
                                                     size_t nvec, V *__restrict__ out)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= nvec) return;
    V s[NP], m[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        s[i] = shares[(size_t)i * nvec + v];
        if (MASK) m[i] = mask[(size_t)i * nvec + v];
    }
    V acc = 0;
#pragma unroll
    for (int i = 0; i < NP; ++i) acc += MASK ? s[i] - m[i] : s[i];
    out[v] = acc;
}

// z_i = c_i + e*b_i + a_i*f (+ e*f for party 0) with e, f opened in registers (Section 4.3).
template <int NP, class V>
__global__ __launch_bounds__(kBlock) void beaver_mul_kernel(const V *__restrict__ x, const V *__restrict__ y,
                                                           const V *__restrict__ a, const V *__restrict__ b,
                                                           const V *__restrict__ c, size_t nvec, V *z)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= nvec) return;
    V xa[NP], yb[NP], av[NP], bv[NP], cv[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        size_t o = (size_t)i * nvec + v;
        xa[i] = x[o]; yb[i] = y[o]; av[i] = a[o]; bv[i] = b[o]; cv[i] = c[o];
    }
    V e = 0, f = 0;
#pragma unroll
    for (int i = 0; i < NP; ++i) { e += xa[i] - av[i]; f += yb[i] - bv[i]; }
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        V bi = bv[i];
        if (i == 0) bi += f;                       // folds the public e*f into party 0's term
        z[(size_t)i * nvec + v] = cv[i] + e * bi + av[i] * f;
    }
}

// Signed probabilistic truncation (Section 4.4); steps as listed at spin_trunc in include/spin.h.
template <int NP, class V>
__global__ __launch_bounds__(kBlock) void trunc_kernel(const V *x, const V *__restrict__ r,
                                                      const V *__restrict__ r_top, const V *__restrict__ r_msb,
                                                      size_t nvec, int f, V *out)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= nvec) return;
    V xv[NP], rt[NP], rm[NP];
    V c = (u64)1 << 62;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        size_t o = (size_t)i * nvec + v;
        xv[i] = x[o]; rt[i] = r_top[o]; rm[i] = r_msb[o];
        c += xv[i] + r[o];
    }
    const u64 topmask = (((u64)1 << (63 - f)) - 1);
    V c_msb = c >> 63;
    V c_top = (c >> f) & topmask;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        V b = rm[i] - 2 * c_msb * rm[i];
        V o = (b << (63 - f)) - rt[i];
        if (i == 0) o += (c_msb << (63 - f)) + c_top - ((u64)1 << (62 - f));
        out[(size_t)i * nvec + v] = o;
    }
}

// y_i = sum_j coef_j in_j,i (+ constant for party 0), then the truncation of trunc_kernel on y when
// TRUNC (Section 4.3 Addition/Scaling; Section 4.4 Polynomial evaluation: one deferred truncation).
// The term loop is a run-time loop; every iteration issues one load per party.
template <int NP, bool TRUNC>
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
        for (int i = 0; i < NP; ++i) y[i] += cf * src[(size_t)i * count + v];
    }
    if (!TRUNC) {
#pragma unroll
        for (int i = 0; i < NP; ++i) out[(size_t)i * count + v] = y[i];
        return;
    }
    u64 rt[NP], rm[NP];
    u64 c = (u64)1 << 62;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        size_t o = (size_t)i * count + v;
        rt[i] = r_top[o]; rm[i] = r_msb[o];
        c += y[i] + r[o];
    }
    const u64 topmask = (((u64)1 << (63 - f)) - 1);
    u64 c_msb = c >> 63;
    u64 c_top = (c >> f) & topmask;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        u64 b = rm[i] - 2 * c_msb * rm[i];
        u64 o = (b << (63 - f)) - rt[i];
        if (i == 0) o += (c_msb << (63 - f)) + c_top - ((u64)1 << (62 - f));
        out[(size_t)i * count + v] = o;
    }
}

inline unsigned grid_for(size_t nvec) { return (unsigned)((nvec + kBlock - 1) / kBlock); }

// Calls fn(integral_constant<int, n>) for the run-time party count.
template <class F> inline void for_party_count(int n, F &&fn)
{
    switch (n) {
    case 1: fn(std::integral_constant<int, 1>()); break;
    case 2: fn(std::integral_constant<int, 2>()); break;
    case 3: fn(std::integral_constant<int, 3>()); break;
    case 4: fn(std::integral_constant<int, 4>()); break;
    case 5: fn(std::integral_constant<int, 5>()); break;
    case 6: fn(std::integral_constant<int, 6>()); break;
    case 7: fn(std::integral_constant<int, 7>()); break;
    default: fn(std::integral_constant<int, 8>()); break;
    }
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
        if (count % 2 == 0)
            share_kernel<NP, u64x2><<<grid_for(count / 2), kBlock, 0, s>>>((const u64x2 *)x, count / 2, keys,
                                                                          (u64x2 *)shares);
        else
            share_kernel<NP, u64><<<grid_for(count), kBlock, 0, s>>>(x, count, keys, shares);
    });
    return check_launch("spin_share");
}

spin_status launch_open(const u64 *shares, const u64 *mask, size_t count, int n, u64 *out, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_OPEN, s);
    for_party_count(n, [&](auto np) {
        constexpr int NP = decltype(np)::value;
        if (kWideLanes && count % 2 == 0) {
            size_t nv = count / 2;
            if (mask)
                open_kernel<NP, true, u64x2><<<grid_for(nv), kBlock, 0, s>>>((const u64x2 *)shares,
                                                                             (const u64x2 *)mask, nv, (u64x2 *)out);
            else
                open_kernel<NP, false, u64x2><<<grid_for(nv), kBlock, 0, s>>>((const u64x2 *)shares, nullptr, nv,
                                                                              (u64x2 *)out);
        } else {
            if (mask) open_kernel<NP, true, u64><<<grid_for(count), kBlock, 0, s>>>(shares, mask, count, out);
            else open_kernel<NP, false, u64><<<grid_for(count), kBlock, 0, s>>>(shares, nullptr, count, out);
        }
    });
    return check_launch("spin_open");
}

spin_status launch_beaver_mul(int n, size_t count, const u64 *x, const u64 *y, const u64 *a, const u64 *b,
                              const u64 *c, u64 *z, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_BEAVER_MUL, s);
    for_party_count(n, [&](auto np) {
        constexpr int NP = decltype(np)::value;
        if (kWideLanes && count % 2 == 0) {
            size_t nv = count / 2;
            beaver_mul_kernel<NP, u64x2><<<grid_for(nv), kBlock, 0, s>>>(
                (const u64x2 *)x, (const u64x2 *)y, (const u64x2 *)a, (const u64x2 *)b, (const u64x2 *)c, nv,
                (u64x2 *)z);
        } else {
            beaver_mul_kernel<NP, u64><<<grid_for(count), kBlock, 0, s>>>(x, y, a, b, c, count, z);
        }
    });
    return check_launch("spin_beaver_mul");
}

spin_status launch_trunc(int n, size_t count, int f, const u64 *x, const u64 *r, const u64 *r_top,
                         const u64 *r_msb, u64 *out, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_TRUNC, s);
    for_party_count(n, [&](auto np) {
        constexpr int NP = decltype(np)::value;
        if (kWideLanes && count % 2 == 0) {
            size_t nv = count / 2;
            trunc_kernel<NP, u64x2><<<grid_for(nv), kBlock, 0, s>>>((const u64x2 *)x, (const u64x2 *)r,
                                                                    (const u64x2 *)r_top, (const u64x2 *)r_msb, nv,
                                                                    f, (u64x2 *)out);
        } else {
            trunc_kernel<NP, u64><<<grid_for(count), kBlock, 0, s>>>(x, r, r_top, r_msb, count, f, out);
        }
    });
    return check_launch("spin_trunc");
}

spin_status launch_lincomb_trunc(int n, size_t count, const LincombTerms &t, u64 constant, int f, const u64 *r,
                                 const u64 *r_top, const u64 *r_msb, u64 *out, hipStream_t s)
{
    KernelTimer timer(SPIN_KERNEL_LINCOMB, s);
    for_party_count(n, [&](auto np) {
        constexpr int NP = decltype(np)::value;
        if (f > 0)
            lincomb_trunc_kernel<NP, true><<<grid_for(count), kBlock, 0, s>>>(t, constant, r, r_top, r_msb, count, f, out);
        else
            lincomb_trunc_kernel<NP, false><<<grid_for(count), kBlock, 0, s>>>(t, constant, nullptr, nullptr, nullptr,
                                                                              count, 0, out);
    });
    return check_launch("spin_lincomb_trunc");
}

}  // namespace spin
