// The C ABI of include/spin.h: argument validation, then dispatch to the
// kernel launchers.  Validation touches no HIP call, so it behaves the same on
// a machine without a GPU.
#include <string.h>

#include <atomic>
#include <mutex>
#include <vector>

#include "common.hpp"

namespace spin {

static thread_local char g_hip_error[256] = "";

void note_hip_error(hipError_t e, const char *where)
{
    snprintf(g_hip_error, sizeof g_hip_error, "%s: %s", where, hipGetErrorString(e));
}

spin_status check_launch(const char *where)
{
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) return SPIN_OK;
    note_hip_error(e, where);
    return SPIN_EHIP;
}

// ---- per-device facts ------------------------------------------------------------
int current_device()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) dev = 0;
    return dev;
}

int compute_units()
{
    static std::atomic<int> cus[kMaxDevices];            // zero-initialised; a race only repeats the query
    const int dev = current_device();
    int v = cus[dev].load(std::memory_order_relaxed);
    if (v == 0) {
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
        cus[dev].store(v, std::memory_order_relaxed);
    }
    return v;
}

spin_status allow_dynamic_lds(const void *kernel, int bytes, OncePerDevice &flags)
{
    static std::mutex m;
    const int dev = current_device();
    std::lock_guard<std::mutex> lock(m);
    if (flags.done[dev]) return SPIN_OK;
    hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) { note_hip_error(e, "hipFuncSetAttribute"); return SPIN_EHIP; }
    flags.done[dev] = 1;
    return SPIN_OK;
}

// ---- optional per-kernel event timing ---------------------------------------
namespace {
struct TimedLaunch { spin_kernel id; hipEvent_t begin, end; };
std::atomic<bool> g_profile{false};
std::mutex g_timed_mutex;
std::vector<TimedLaunch> g_timed;
}  // namespace

// > 0 while this thread is inside an entry point that must not allocate: no event objects are created then
static thread_local int g_no_timing = 0;
struct NoTimingScope { NoTimingScope() { ++g_no_timing; } ~NoTimingScope() { --g_no_timing; } };

KernelTimer::KernelTimer(spin_kernel id_, hipStream_t s) : id(id_), stream(s), begin(nullptr), active(false)
{
    (void)hipGetLastError();                             // a stale error of an earlier call is not this launch's
    if (g_no_timing > 0 || !g_profile.load(std::memory_order_relaxed)) return;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) {
        (void)hipGetLastError();
        return;
    }
    if (hipEventCreate(&begin) != hipSuccess) return;
    active = hipEventRecord(begin, stream) == hipSuccess;
    if (!active) (void)hipEventDestroy(begin);
}

KernelTimer::~KernelTimer()
{
    if (!active) return;
    hipEvent_t end;
    if (hipEventCreate(&end) != hipSuccess) { (void)hipEventDestroy(begin); return; }
    if (hipEventRecord(end, stream) != hipSuccess) { (void)hipEventDestroy(begin); (void)hipEventDestroy(end); return; }
    std::lock_guard<std::mutex> lock(g_timed_mutex);
    g_timed.push_back({id, begin, end});
}

namespace {
inline bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }
inline bool bad_ptr(const void *p) { return p == nullptr || !aligned16(p); }
inline bool bad_n(int n) { return n < 1 || n > SPIN_MAX_PARTIES; }
// element counts are limited so that n * count * 8 and the grid size stay in range
constexpr size_t kMaxCount = (size_t)1 << 38;
}  // namespace
}  // namespace spin

using namespace spin;

extern "C" {

spin_status spin_random(uint64_t *out, size_t count, uint64_t seed, uint64_t stream_id, uint64_t party,
                        uint64_t first_idx, spin_stream stream)
{
    if (bad_ptr(out) || count == 0) return SPIN_EINVAL;
    if (count > kMaxCount) return SPIN_ERANGE;
    return launch_random(out, count, stream_key(seed, stream_id, party), first_idx, (hipStream_t)stream);
}

spin_status spin_share(const uint64_t *x, size_t count, int n, uint64_t seed, uint64_t stream_id,
                       uint64_t *shares, spin_stream stream)
{
    if (bad_ptr(x) || bad_ptr(shares) || bad_n(n) || count == 0) return SPIN_EINVAL;
    if (count > kMaxCount) return SPIN_ERANGE;
    PartyKeys keys;
    for (int i = 0; i < SPIN_MAX_PARTIES; ++i) keys.key[i] = stream_key(seed, stream_id, (u64)i);
    return launch_share(x, count, n, keys, shares, (hipStream_t)stream);
}

spin_status spin_open(const uint64_t *shares, const uint64_t *mask, size_t count, int n, uint64_t *out,
                      spin_stream stream)
{
    if (bad_ptr(shares) || bad_ptr(out) || (mask && !aligned16(mask)) || bad_n(n) || count == 0)
        return SPIN_EINVAL;
    if (count > kMaxCount) return SPIN_ERANGE;
    return launch_open(shares, mask, count, n, out, (hipStream_t)stream);
}

static spin_status check_matmul_dims(int n, int batch, int M, int N, int K)
{
    if (bad_n(n) || batch < 1 || M < 1 || N < 1 || K < 1) return SPIN_EINVAL;
    // every operand must stay below 2^38 elements per party and the launch grids within HIP's limits
    const size_t lim = kMaxCount;
    if ((size_t)batch * M * K > lim || (size_t)batch * K * N > lim || (size_t)batch * M * N > lim)
        return SPIN_ERANGE;
    if ((long)n * batch > 65535) return SPIN_ERANGE;
    if (M > (1 << 24) || N > (1 << 24) || K > (1 << 24)) return SPIN_ERANGE;
    return SPIN_OK;
}

size_t spin_beaver_matmul_workspace_bytes(int n, int batch, int M, int N, int K, int path)
{
    if (check_matmul_dims(n, batch, M, N, K) != SPIN_OK) return 0;
    if (path == SPIN_GEMM_LIMB_MFMA) return limb_workspace_bytes(n, batch, M, N, K);
    if (path == SPIN_GEMM_VALU) return valu_workspace_bytes(n, batch, M, N, K, 8);
    return 0;
}

// Everything spin_beaver_matmul checks except the workspace; touches no HIP call.
static spin_status check_matmul64(int n, int batch, int M, int N, int K, const uint64_t *X, const uint64_t *Y,
                                  const uint64_t *A, const uint64_t *B, const uint64_t *C, uint64_t *Z,
                                  int path)
{
    if (bad_ptr(X) || bad_ptr(Y) || bad_ptr(A) || bad_ptr(B) || bad_ptr(C) || bad_ptr(Z)) return SPIN_EINVAL;
    if (path != SPIN_GEMM_LIMB_MFMA && path != SPIN_GEMM_VALU) return SPIN_EINVAL;
    return check_matmul_dims(n, batch, M, N, K);
}

static spin_status beaver_matmul64(int n, int batch, int M, int N, int K, const uint64_t *X, const uint64_t *Y,
                                   const uint64_t *A, const uint64_t *B, const uint64_t *C, uint64_t *Z,
                                   int path, void *workspace, size_t workspace_bytes, spin_stream stream,
                                   bool y_transposed)
{
    spin_status st = check_matmul64(n, batch, M, N, K, X, Y, A, B, C, Z, path);
    if (st != SPIN_OK) return st;
    const size_t need = spin_beaver_matmul_workspace_bytes(n, batch, M, N, K, path);
    if (workspace == nullptr || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < need)
        return SPIN_EWORKSPACE;
    MatmulArgs a{n, batch, M, N, K, X, Y, A, B, C, Z, workspace, y_transposed};
    return path == SPIN_GEMM_LIMB_MFMA ? launch_matmul_limb(a, (hipStream_t)stream)
                                       : launch_matmul_valu(a, (hipStream_t)stream);
}

spin_status spin_beaver_matmul(int n, int batch, int M, int N, int K, const uint64_t *X, const uint64_t *Y,
                               const uint64_t *A, const uint64_t *B, const uint64_t *C, uint64_t *Z,
                               int path, void *workspace, size_t workspace_bytes, spin_stream stream)
{
    return beaver_matmul64(n, batch, M, N, K, X, Y, A, B, C, Z, path, workspace, workspace_bytes, stream, false);
}

spin_status spin_beaver_matmul_nt(int n, int batch, int M, int N, int K, const uint64_t *X, const uint64_t *Yt,
                                  const uint64_t *A, const uint64_t *Bt, const uint64_t *C, uint64_t *Z,
                                  int path, void *workspace, size_t workspace_bytes, spin_stream stream)
{
    return beaver_matmul64(n, batch, M, N, K, X, Yt, A, Bt, C, Z, path, workspace, workspace_bytes, stream, true);
}

size_t spin_beaver_matmul_grouped_workspace_bytes(int n, int groups, const spin_matmul_group *desc, int path)
{
    if (desc == nullptr || groups < 1 || groups > SPIN_MAX_GROUPS) return 0;
    size_t largest = 0, sum = 0;
    for (int g = 0; g < groups; ++g) {
        const size_t b = spin_beaver_matmul_workspace_bytes(n, desc[g].batch, desc[g].M, desc[g].N, desc[g].K, path);
        if (b == 0) return 0;
        if (b > largest) largest = b;
        sum += b;
    }
    // the limb path packs every group before the first GEMM runs, so all fragment stores exist at once
    return path == SPIN_GEMM_LIMB_MFMA ? sum : largest;
}

spin_status spin_beaver_matmul_grouped(int n, int groups, const spin_matmul_group *desc, int path,
                                       void *workspace, size_t workspace_bytes, spin_stream stream)
{
    if (desc == nullptr || groups < 1 || groups > SPIN_MAX_GROUPS) return SPIN_EINVAL;
    if (path != SPIN_GEMM_LIMB_MFMA && path != SPIN_GEMM_VALU) return SPIN_EINVAL;
    for (int g = 0; g < groups; ++g) {                   // everything is checked before anything is launched
        const spin_matmul_group &d = desc[g];
        if (bad_ptr(d.X) || bad_ptr(d.Y) || bad_ptr(d.A) || bad_ptr(d.B) || bad_ptr(d.C) || bad_ptr(d.Z)) return SPIN_EINVAL;
        spin_status st = check_matmul_dims(n, d.batch, d.M, d.N, d.K);
        if (st != SPIN_OK) return st;
    }
    const size_t need = spin_beaver_matmul_grouped_workspace_bytes(n, groups, desc, path);
    if (workspace == nullptr || ((uintptr_t)workspace & 255) != 0 || need == 0 || workspace_bytes < need)
        return SPIN_EWORKSPACE;
    if (path == SPIN_GEMM_LIMB_MFMA) {
        MatmulArgs args[SPIN_MAX_GROUPS];
        for (int g = 0; g < groups; ++g) {
            const spin_matmul_group &d = desc[g];
            args[g] = MatmulArgs{n, d.batch, d.M, d.N, d.K, d.X, d.Y, d.A, d.B, d.C, d.Z, nullptr, d.y_transposed != 0};
        }
        const spin_status st = launch_matmul_limb_grouped(n, groups, args, workspace, (hipStream_t)stream);
        if (st != SPIN_ERANGE) return st;                // SPIN_ERANGE: a group does not fit a shared launch, nothing was launched
    }
    for (int g = 0; g < groups; ++g) {
        const spin_matmul_group &d = desc[g];
        spin_status st = beaver_matmul64(n, d.batch, d.M, d.N, d.K, d.X, d.Y, d.A, d.B, d.C, d.Z, path, workspace,
                                         workspace_bytes, stream, d.y_transposed != 0);
        if (st != SPIN_OK) return st;
    }
    return SPIN_OK;
}

}  // extern "C"

// ---- the entry point that allocates nothing ----------------------------------------------------
// The workspace of spin_beaver_matmul_static lives in the library's own device image: every GPU the
// library runs on holds one copy of this array, at its own address, until the process ends.  In host
// code the array's name is only a handle for the runtime's symbol lookup, never a device address: the
// address is asked for once per device (with that device current) and only that pointer is handed to
// kernels.
namespace {
static __device__ __align__(256) unsigned char scratch[SPIN_STATIC_WORKSPACE_BYTES];
void *g_scratch_ptr[spin::kMaxDevices];                  // device address of `scratch`, per device
std::mutex g_scratch_mutex;

spin_status static_workspace(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { note_hip_error(e, "hipGetDevice"); return SPIN_EHIP; }
    if (dev < 0 || dev >= spin::kMaxDevices) { note_hip_error(hipErrorInvalidDevice, "spin_beaver_matmul_static"); return SPIN_EHIP; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || ptr == nullptr) {
            note_hip_error(e != hipSuccess ? e : hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch)");
            return SPIN_EHIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SPIN_OK;
}
}  // namespace

extern "C" {

spin_status spin_beaver_matmul_static(int n, int batch, int M, int N, int K, const uint64_t *X, const uint64_t *Y,
                                      const uint64_t *A, const uint64_t *B, const uint64_t *C, uint64_t *Z,
                                      int path, spin_stream stream)
{
    spin_status st = check_matmul64(n, batch, M, N, K, X, Y, A, B, C, Z, path);
    if (st != SPIN_OK) return st;
    const size_t need = spin_beaver_matmul_workspace_bytes(n, batch, M, N, K, path);
    if (need == 0 || need > (size_t)SPIN_STATIC_WORKSPACE_BYTES) return SPIN_EWORKSPACE;
    void *ws = nullptr;
    st = static_workspace(&ws);
    if (st != SPIN_OK) return st;
    NoTimingScope no_events;                             // event timing would create event objects
    // Nothing in the workspace has to start at zero: the pack kernels (limb path) and the opening of E and F
    // (baseline path) overwrite every byte a later kernel reads, padding included, on every call.
    MatmulArgs a{n, batch, M, N, K, X, Y, A, B, C, Z, ws, false};
    return path == SPIN_GEMM_LIMB_MFMA ? launch_matmul_limb(a, (hipStream_t)stream)
                                       : launch_matmul_valu(a, (hipStream_t)stream);
}

spin_status spin_beaver_mul(int n, size_t count, const uint64_t *x, const uint64_t *y, const uint64_t *a,
                            const uint64_t *b, const uint64_t *c, uint64_t *z, spin_stream stream)
{
    if (bad_ptr(x) || bad_ptr(y) || bad_ptr(a) || bad_ptr(b) || bad_ptr(c) || bad_ptr(z) || bad_n(n) || count == 0)
        return SPIN_EINVAL;
    if (count > kMaxCount) return SPIN_ERANGE;
    return launch_beaver_mul(n, count, x, y, a, b, c, z, (hipStream_t)stream);
}

spin_status spin_beaver_mul_trunc(int n, size_t count, int f, const uint64_t *x, const uint64_t *y, const uint64_t *a,
                                  const uint64_t *b, const uint64_t *c, const uint64_t *r, const uint64_t *r_top,
                                  const uint64_t *r_msb, uint64_t *out, spin_stream stream)
{
    if (bad_ptr(x) || bad_ptr(y) || bad_ptr(a) || bad_ptr(b) || bad_ptr(c) || bad_ptr(r) || bad_ptr(r_top) ||
        bad_ptr(r_msb) || bad_ptr(out) || bad_n(n) || count == 0)
        return SPIN_EINVAL;
    if (f < 1 || f > 61) return SPIN_EINVAL;
    if (count > kMaxCount) return SPIN_ERANGE;
    return launch_beaver_mul_trunc(n, count, f, x, y, a, b, c, r, r_top, r_msb, out, (hipStream_t)stream);
}

spin_status spin_beaver_mul_bcast(int n, size_t outer, size_t mid, size_t inner, int over_inner, const uint64_t *x,
                                  const uint64_t *y, const uint64_t *a, const uint64_t *b, const uint64_t *c,
                                  uint64_t *z, spin_stream stream)
{
    if (bad_ptr(x) || bad_ptr(y) || bad_ptr(a) || bad_ptr(b) || bad_ptr(c) || bad_ptr(z) || bad_n(n)) return SPIN_EINVAL;
    if (outer == 0 || mid == 0 || inner == 0) return SPIN_EINVAL;
    if (outer > kMaxCount || mid > kMaxCount || inner > kMaxCount || outer * mid > kMaxCount ||
        outer * mid * inner > kMaxCount)
        return SPIN_ERANGE;
    return launch_beaver_mul_bcast(n, outer, mid, inner, over_inner != 0, x, y, a, b, c, z, (hipStream_t)stream);
}

spin_status spin_trunc(int n, size_t count, int f, const uint64_t *x, const uint64_t *r, const uint64_t *r_top,
                       const uint64_t *r_msb, uint64_t *out, spin_stream stream)
{
    if (bad_ptr(x) || bad_ptr(r) || bad_ptr(r_top) || bad_ptr(r_msb) || bad_ptr(out) || bad_n(n) || count == 0)
        return SPIN_EINVAL;
    if (f < 1 || f > 61) return SPIN_EINVAL;
    if (count > kMaxCount) return SPIN_ERANGE;
    return launch_trunc(n, count, f, x, r, r_top, r_msb, out, (hipStream_t)stream);
}

void spin_profile_enable(int on) { g_profile.store(on != 0); }

void spin_profile_reset(void)
{
    std::lock_guard<std::mutex> lock(g_timed_mutex);
    for (auto &t : g_timed) { (void)hipEventDestroy(t.begin); (void)hipEventDestroy(t.end); }
    g_timed.clear();
}

spin_status spin_profile_read(int kernel, double *total_ms, unsigned *launches)
{
    if (!total_ms || !launches || kernel < 0 || kernel >= SPIN_KERNEL_COUNT) return SPIN_EINVAL;
    double sum = 0.0;
    unsigned cnt = 0;
    std::lock_guard<std::mutex> lock(g_timed_mutex);
    for (auto &t : g_timed) {
        if (t.id != kernel) continue;
        hipError_t e = hipEventSynchronize(t.end);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, t.begin, t.end);
        if (e != hipSuccess) { note_hip_error(e, "spin_profile_read"); return SPIN_EHIP; }
        sum += ms;
        ++cnt;
    }
    *total_ms = sum;
    *launches = cnt;
    return SPIN_OK;
}

spin_status spin_bshare(const uint64_t *x, size_t count, int n, uint64_t seed, uint64_t stream_id,
                        uint64_t *shares, spin_stream stream)
{
    if (bad_ptr(x) || bad_ptr(shares) || bad_n(n) || count == 0) return SPIN_EINVAL;
    if (count > kMaxCount) return SPIN_ERANGE;
    PartyKeys keys;
    for (int i = 0; i < SPIN_MAX_PARTIES; ++i) keys.key[i] = stream_key(seed, stream_id, (u64)i);
    return launch_bshare(x, count, n, keys, shares, (hipStream_t)stream);
}

spin_status spin_bopen(const uint64_t *shares, const uint64_t *mask, size_t count, int n, uint64_t *out,
                       spin_stream stream)
{
    if (bad_ptr(shares) || bad_ptr(out) || (mask && !aligned16(mask)) || bad_n(n) || count == 0)
        return SPIN_EINVAL;
    if (count > kMaxCount) return SPIN_ERANGE;
    return launch_bopen(shares, mask, count, n, out, (hipStream_t)stream);
}

spin_status spin_beaver_and(int n, size_t count, const uint64_t *x, const uint64_t *y, const uint64_t *a,
                            const uint64_t *b, const uint64_t *c, uint64_t *z, spin_stream stream)
{
    if (bad_ptr(x) || bad_ptr(y) || bad_ptr(a) || bad_ptr(b) || bad_ptr(c) || bad_ptr(z) || bad_n(n) || count == 0)
        return SPIN_EINVAL;
    if (count > kMaxCount) return SPIN_ERANGE;
    return launch_beaver_and(n, count, x, y, a, b, c, z, (hipStream_t)stream);
}

spin_status spin_lincomb_trunc(int n, size_t count, int terms, const uint64_t *const *in, const uint64_t *coef,
                               uint64_t constant, int f, const uint64_t *r, const uint64_t *r_top,
                               const uint64_t *r_msb, uint64_t *out, spin_stream stream)
{
    if (in == nullptr || coef == nullptr || bad_ptr(out) || bad_n(n) || count == 0) return SPIN_EINVAL;
    if (terms < 1 || terms > SPIN_MAX_TERMS || f < 0 || f > 61) return SPIN_EINVAL;
    if (f > 0 && (bad_ptr(r) || bad_ptr(r_top) || bad_ptr(r_msb))) return SPIN_EINVAL;
    LincombTerms t;
    t.terms = terms;
    for (int j = 0; j < SPIN_MAX_TERMS; ++j) { t.in[j] = nullptr; t.coef[j] = 0; }
    for (int j = 0; j < terms; ++j) {
        if (bad_ptr(in[j])) return SPIN_EINVAL;
        t.in[j] = in[j];
        t.coef[j] = coef[j];
    }
    if (count > kMaxCount) return SPIN_ERANGE;
    return launch_lincomb_trunc(n, count, t, constant, f, r, r_top, r_msb, out, (hipStream_t)stream);
}

// ---- Z_2^128 --------------------------------------------------------------------------------------
static inline const u128 *r128(const uint64_t *p) { return (const u128 *)p; }
static inline u128 *r128(uint64_t *p) { return (u128 *)p; }

spin_status spin128_share(const uint64_t *x, size_t count, int n, uint64_t seed, uint64_t stream_id,
                          uint64_t *shares, spin_stream stream)
{
    if (bad_ptr(x) || bad_ptr(shares) || bad_n(n) || count == 0) return SPIN_EINVAL;
    if (count > kMaxCount / 2) return SPIN_ERANGE;
    PartyKeys keys;
    for (int i = 0; i < SPIN_MAX_PARTIES; ++i) keys.key[i] = stream_key(seed, stream_id, (u64)i);
    return launch_share128(r128(x), count, n, keys, r128(shares), (hipStream_t)stream);
}

spin_status spin128_open(const uint64_t *shares, const uint64_t *mask, size_t count, int n, uint64_t *out,
                         spin_stream stream)
{
    if (bad_ptr(shares) || bad_ptr(out) || (mask && !aligned16(mask)) || bad_n(n) || count == 0)
        return SPIN_EINVAL;
    if (count > kMaxCount / 2) return SPIN_ERANGE;
    return launch_open<u128>(r128(shares), r128(mask), count, n, r128(out), (hipStream_t)stream);
}

size_t spin128_beaver_matmul_workspace_bytes(int n, int batch, int M, int N, int K, int path)
{
    if (check_matmul_dims(n, batch, M, N, K) != SPIN_OK) return 0;
    if (path == SPIN_GEMM_LIMB_MFMA) return limb128_workspace_bytes(n, batch, M, N, K);
    if (path == SPIN_GEMM_VALU) return valu_workspace_bytes(n, batch, M, N, K, 16);
    return 0;
}

spin_status spin128_beaver_matmul(int n, int batch, int M, int N, int K, const uint64_t *X, const uint64_t *Y,
                                  const uint64_t *A, const uint64_t *B, const uint64_t *C, uint64_t *Z,
                                  int path, void *workspace, size_t workspace_bytes, spin_stream stream)
{
    if (bad_ptr(X) || bad_ptr(Y) || bad_ptr(A) || bad_ptr(B) || bad_ptr(C) || bad_ptr(Z)) return SPIN_EINVAL;
    if (path != SPIN_GEMM_LIMB_MFMA && path != SPIN_GEMM_VALU) return SPIN_EINVAL;
    spin_status st = check_matmul_dims(n, batch, M, N, K);
    if (st != SPIN_OK) return st;
    const size_t need = spin128_beaver_matmul_workspace_bytes(n, batch, M, N, K, path);
    if (workspace == nullptr || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < need)
        return SPIN_EWORKSPACE;
    MatmulArgs128 a{n, batch, M, N, K, r128(X), r128(Y), r128(A), r128(B), r128(C), r128(Z), workspace, false};
    return path == SPIN_GEMM_LIMB_MFMA ? launch_matmul_limb128(a, (hipStream_t)stream)
                                       : launch_matmul_valu<u128>(a, (hipStream_t)stream);
}

spin_status spin128_beaver_mul(int n, size_t count, const uint64_t *x, const uint64_t *y, const uint64_t *a,
                               const uint64_t *b, const uint64_t *c, uint64_t *z, spin_stream stream)
{
    if (bad_ptr(x) || bad_ptr(y) || bad_ptr(a) || bad_ptr(b) || bad_ptr(c) || bad_ptr(z) || bad_n(n) || count == 0)
        return SPIN_EINVAL;
    if (count > kMaxCount / 2) return SPIN_ERANGE;
    return launch_beaver_mul<u128>(n, count, r128(x), r128(y), r128(a), r128(b), r128(c), r128(z), (hipStream_t)stream);
}

spin_status spin128_trunc(int n, size_t count, int f, const uint64_t *x, const uint64_t *r, const uint64_t *r_top,
                          const uint64_t *r_msb, uint64_t *out, spin_stream stream)
{
    if (bad_ptr(x) || bad_ptr(r) || bad_ptr(r_top) || bad_ptr(r_msb) || bad_ptr(out) || bad_n(n) || count == 0)
        return SPIN_EINVAL;
    if (f < 1 || f > 125) return SPIN_EINVAL;
    if (count > kMaxCount / 2) return SPIN_ERANGE;
    return launch_trunc<u128>(n, count, f, r128(x), r128(r), r128(r_top), r128(r_msb), r128(out), (hipStream_t)stream);
}

// ---- Z_2^32 --------------------------------------------------------------------------------
spin_status spin32_share(const uint32_t *x, size_t count, int n, uint64_t seed, uint64_t stream_id,
                         uint32_t *shares, spin_stream stream)
{
    if (bad_ptr(x) || bad_ptr(shares) || bad_n(n) || count == 0) return SPIN_EINVAL;
    if (count > kMaxCount) return SPIN_ERANGE;
    PartyKeys keys;
    for (int i = 0; i < SPIN_MAX_PARTIES; ++i) keys.key[i] = stream_key(seed, stream_id, (u64)i);
    return launch_share32(x, count, n, keys, shares, (hipStream_t)stream);
}

spin_status spin32_open(const uint32_t *shares, const uint32_t *mask, size_t count, int n, uint32_t *out,
                        spin_stream stream)
{
    if (bad_ptr(shares) || bad_ptr(out) || (mask && !aligned16(mask)) || bad_n(n) || count == 0)
        return SPIN_EINVAL;
    if (count > kMaxCount) return SPIN_ERANGE;
    return launch_open<u32>(shares, mask, count, n, out, (hipStream_t)stream);
}

size_t spin32_beaver_matmul_workspace_bytes(int n, int batch, int M, int N, int K, int path)
{
    if (check_matmul_dims(n, batch, M, N, K) != SPIN_OK) return 0;
    if (path == SPIN_GEMM_LIMB_MFMA) return limb32_workspace_bytes(n, batch, M, N, K);
    if (path == SPIN_GEMM_VALU) return valu_workspace_bytes(n, batch, M, N, K, 4);
    return 0;
}

spin_status spin32_beaver_matmul(int n, int batch, int M, int N, int K, const uint32_t *X, const uint32_t *Y,
                                 const uint32_t *A, const uint32_t *B, const uint32_t *C, uint32_t *Z,
                                 int path, void *workspace, size_t workspace_bytes, spin_stream stream)
{
    if (bad_ptr(X) || bad_ptr(Y) || bad_ptr(A) || bad_ptr(B) || bad_ptr(C) || bad_ptr(Z)) return SPIN_EINVAL;
    if (path != SPIN_GEMM_LIMB_MFMA && path != SPIN_GEMM_VALU) return SPIN_EINVAL;
    spin_status st = check_matmul_dims(n, batch, M, N, K);
    if (st != SPIN_OK) return st;
    const size_t need = spin32_beaver_matmul_workspace_bytes(n, batch, M, N, K, path);
    if (workspace == nullptr || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < need)
        return SPIN_EWORKSPACE;
    MatmulArgs32 a{n, batch, M, N, K, X, Y, A, B, C, Z, workspace, false};
    return path == SPIN_GEMM_LIMB_MFMA ? launch_matmul_limb32(a, (hipStream_t)stream)
                                       : launch_matmul_valu<u32>(a, (hipStream_t)stream);
}

spin_status spin32_beaver_mul(int n, size_t count, const uint32_t *x, const uint32_t *y, const uint32_t *a,
                              const uint32_t *b, const uint32_t *c, uint32_t *z, spin_stream stream)
{
    if (bad_ptr(x) || bad_ptr(y) || bad_ptr(a) || bad_ptr(b) || bad_ptr(c) || bad_ptr(z) || bad_n(n) || count == 0)
        return SPIN_EINVAL;
    if (count > kMaxCount) return SPIN_ERANGE;
    return launch_beaver_mul<u32>(n, count, x, y, a, b, c, z, (hipStream_t)stream);
}

spin_status spin32_trunc(int n, size_t count, int f, const uint32_t *x, const uint32_t *r, const uint32_t *r_top,
                         const uint32_t *r_msb, uint32_t *out, spin_stream stream)
{
    if (bad_ptr(x) || bad_ptr(r) || bad_ptr(r_top) || bad_ptr(r_msb) || bad_ptr(out) || bad_n(n) || count == 0)
        return SPIN_EINVAL;
    if (f < 1 || f > 29) return SPIN_EINVAL;
    if (count > kMaxCount) return SPIN_ERANGE;
    return launch_trunc<u32>(n, count, f, x, r, r_top, r_msb, out, (hipStream_t)stream);
}

spin_status spin_cast_64_to_32(const uint64_t *in, size_t count, uint32_t *out, spin_stream stream)
{
    if (bad_ptr(in) || bad_ptr(out) || count == 0) return SPIN_EINVAL;
    if (count > kMaxCount) return SPIN_ERANGE;
    return launch_cast_low(in, count, out, (hipStream_t)stream);
}

spin_status spin_probe_mfma(const uint64_t *operands, int blocks, int iters, uint64_t *sink, spin_stream stream)
{
    if (bad_ptr(operands) || bad_ptr(sink)) return SPIN_EINVAL;
    if (blocks < 1 || blocks > (1 << 20) || iters < 1 || iters > (1 << 20)) return SPIN_EINVAL;
    return launch_mfma_probe(operands, blocks, iters, sink, (hipStream_t)stream);
}

const char *spin_status_string(int status)
{
    switch (status) {
    case SPIN_OK: return "ok";
    case SPIN_EINVAL: return "invalid argument";
    case SPIN_ERANGE: return "size out of range";
    case SPIN_EWORKSPACE: return "workspace missing, misaligned or too small";
    case SPIN_EHIP: return "HIP launch failure";
    }
    return "unknown status";
}

const char *spin_last_hip_error(void) { return g_hip_error; }

}  // extern "C"
