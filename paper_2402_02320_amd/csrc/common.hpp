// Shared host/device helpers of the gfx950 library: the counter generator,
// 16-byte ring vectors, launch bookkeeping.  Internal; the public surface is
// include/spin.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <type_traits>

#include "../../include/spin_bench.h"

namespace spin {

typedef uint64_t u64;
typedef uint32_t u32;             // ring Z_2^32 (the Fixed32 representation of Section 7.1)
typedef u64 u64x2 __attribute__((ext_vector_type(2)));
typedef u32 u32x2 __attribute__((ext_vector_type(2)));
typedef u32 u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned __int128 u128;   // ring Z_2^128: 16 bytes, little-endian (low word first)

// ---- counter generator (specified in include/spin.h at spin_random) --------
__host__ __device__ inline u64 mix64(u64 z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}
__host__ __device__ inline u64 absorb(u64 h, u64 v) { return mix64(h + (v + 1) * 0x9E3779B97F4A7C15ull); }
// Everything of rand64 that does not depend on the element index.
inline u64 stream_key(u64 seed, u64 stream_id, u64 party)
{
    return absorb(absorb(absorb(0, seed), stream_id), party);
}

struct PartyKeys { u64 key[SPIN_MAX_PARTIES]; };

// Calls fn(std::integral_constant<int, n>) for the run-time party count, so that kernels can be
// templated on it (all of a thread's per-party loads are then issued before the first use).
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

// ---- launch bookkeeping ------------------------------------------------------
void note_hip_error(hipError_t e, const char *where);
// Returns SPIN_OK or records the launch error and returns SPIN_EHIP.  Only errors raised since the
// enclosing KernelTimer was constructed are seen (it discards whatever an earlier, unrelated HIP call left).
spin_status check_launch(const char *where);

// Every launcher constructs one before its launches.  It clears the runtime's sticky last-error slot, so
// that check_launch reports this launch only, and, when profiling is enabled and the stream is not being
// captured into a graph, brackets the launches made during its lifetime with a HIP event pair.
struct KernelTimer {
    KernelTimer(spin_kernel id, hipStream_t s);
    ~KernelTimer();
    spin_kernel id; hipStream_t stream; hipEvent_t begin; bool active;
};

// Per-device facts and one-time set-up, indexed by the current device.
constexpr int kMaxDevices = 64;
int current_device();                 // hipGetDevice, clamped to [0, kMaxDevices)
int compute_units();                  // of the current device (256 when the runtime cannot say)
// Raises a kernel's dynamic-LDS limit once per device; `done` is that kernel's per-device flag array.
struct OncePerDevice { unsigned char done[kMaxDevices]; };
spin_status allow_dynamic_lds(const void *kernel, int bytes, OncePerDevice &flags);

// ---- internal launchers (defined in the .hip files) -------------------------
spin_status launch_random(u64 *out, size_t count, u64 key, u64 first_idx, hipStream_t s);
spin_status launch_share(const u64 *x, size_t count, int n, const PartyKeys &keys, u64 *shares, hipStream_t s);
// T = u32, u64 or u128 (instantiated in elementwise.hip)
template <class T> spin_status launch_open(const T *shares, const T *mask, size_t count, int n, T *out, hipStream_t s);
template <class T>
spin_status launch_beaver_mul(int n, size_t count, const T *x, const T *y, const T *a, const T *b, const T *c, T *z,
                              hipStream_t s);
spin_status launch_beaver_mul_trunc(int n, size_t count, int f, const u64 *x, const u64 *y, const u64 *a, const u64 *b,
                                    const u64 *c, const u64 *r, const u64 *r_top, const u64 *r_msb, u64 *out,
                                    hipStream_t s);
spin_status launch_beaver_mul_bcast(int n, size_t outer, size_t mid, size_t inner, bool over_inner, const u64 *x,
                                    const u64 *y, const u64 *a, const u64 *b, const u64 *c, u64 *z, hipStream_t s);
template <class T>
spin_status launch_trunc(int n, size_t count, int f, const T *x, const T *r, const T *r_top, const T *r_msb, T *out,
                         hipStream_t s);
spin_status launch_share32(const u32 *x, size_t count, int n, const PartyKeys &keys, u32 *shares, hipStream_t s);
spin_status launch_cast_low(const u64 *in, size_t count, u32 *out, hipStream_t s);
spin_status launch_share128(const u128 *x, size_t count, int n, const PartyKeys &keys, u128 *shares, hipStream_t s);

spin_status launch_bshare(const u64 *x, size_t count, int n, const PartyKeys &keys, u64 *shares, hipStream_t s);
spin_status launch_bopen(const u64 *shares, const u64 *mask, size_t count, int n, u64 *out, hipStream_t s);
spin_status launch_beaver_and(int n, size_t count, const u64 *x, const u64 *y, const u64 *a, const u64 *b,
                              const u64 *c, u64 *z, hipStream_t s);
struct LincombTerms { const u64 *in[SPIN_MAX_TERMS]; u64 coef[SPIN_MAX_TERMS]; int terms; };
spin_status launch_lincomb_trunc(int n, size_t count, const LincombTerms &t, u64 constant, int f, const u64 *r,
                                 const u64 *r_top, const u64 *r_msb, u64 *out, hipStream_t s);

template <class T> struct MatmulArgsT {
    int n, batch, M, N, K;
    const T *X, *Y, *A, *B, *C;
    T *Z;
    void *workspace;
    bool y_transposed;     // Y and B are stored [n][batch][N][K] instead of [n][batch][K][N]
};
typedef MatmulArgsT<u64> MatmulArgs;
typedef MatmulArgsT<u128> MatmulArgs128;
typedef MatmulArgsT<u32> MatmulArgs32;
// elem_bytes = 4 (Z_2^32), 8 (Z_2^64) or 16 (Z_2^128)
size_t valu_workspace_bytes(int n, int batch, int M, int N, int K, int elem_bytes);
template <class T> spin_status launch_matmul_valu(const MatmulArgsT<T> &a, hipStream_t s);
size_t limb_workspace_bytes(int n, int batch, int M, int N, int K);
spin_status launch_matmul_limb(const MatmulArgs &a, hipStream_t s);
// groups of different shapes in shared launches (a[g].workspace is ignored: every group gets its own part of `workspace`)
size_t limb_grouped_workspace_bytes(int n, int groups, const MatmulArgs *a);
spin_status launch_matmul_limb_grouped(int n, int groups, const MatmulArgs *a, void *workspace, hipStream_t s);
size_t limb32_workspace_bytes(int n, int batch, int M, int N, int K);
spin_status launch_matmul_limb32(const MatmulArgs32 &a, hipStream_t s);
spin_status launch_mfma_probe(const u64 *operands, int blocks, int iters, u64 *sink, hipStream_t s);
size_t limb128_workspace_bytes(int n, int batch, int M, int N, int K);
spin_status launch_matmul_limb128(const MatmulArgs128 &a, hipStream_t s);

}  // namespace spin
