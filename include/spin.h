/*
 * spin.h -- C ABI of the MI355X (gfx950) library for the per-party local work
 * of additive-secret-sharing multiplication over the ring Z_2^64:
 * sharing, opening, the Beaver-triple share update for matrix and elementwise
 * products, and fixed-point truncation (spin_share, spin_open,
 * spin_beaver_matmul, spin_beaver_mul, spin_trunc).  Further down: the same
 * over Z_2^32 and Z_2^128 (spin32_*, spin128_*), binary shares (spin_b*),
 * and a public linear combination with fused truncation.  Measurement aids
 * (per-kernel event timing, an MFMA rate probe) are declared in spin_bench.h.
 *
 * Conventions that hold for every entry point
 * -------------------------------------------
 *  - Ring elements are uint64_t unless a section says otherwise; all arithmetic
 *    wraps mod 2^64.  Read as signed they are the range [-2^63, 2^63-1] of
 *    Section 4.1 (Notations).
 *  - All n parties live on the one GPU.  Share tensors are party-major:
 *    T[i] is party i's share, contiguous, so a tensor of `count` elements is
 *    laid out [n][count].  Party 0 is the paper's party 1: it holds residual
 *    shares and adds every public term.
 *  - Every data pointer is a DEVICE pointer, 16-byte aligned (the widest vector
 *    access any kernel makes; workspaces 256-byte), owned by the caller; the
 *    entry points of this header never allocate, free or keep a pointer.
 *    Buffers must not overlap unless a function says an output may alias an
 *    input.
 *  - Calls are asynchronous: work is enqueued on `stream` (a hipStream_t; NULL
 *    is the default stream) and the function returns without synchronising.
 *  - Errors are return codes.  Arguments are validated before anything is
 *    launched, so SPIN_EINVAL / SPIN_ERANGE / SPIN_EWORKSPACE never leave
 *    partial work behind.  Nothing throws across the boundary.
 *  - 1 <= n <= SPIN_MAX_PARTIES.
 */
#ifndef SPIN_H
#define SPIN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPIN_MAX_PARTIES 8

typedef enum {
    SPIN_OK = 0,
    SPIN_EINVAL = 1,     /* null pointer, n out of range, non-positive size, f out of range, misaligned */
    SPIN_ERANGE = 2,     /* a size whose element count or padded extent does not fit the index types  */
    SPIN_EWORKSPACE = 3, /* workspace missing or smaller than spin_beaver_matmul_workspace_bytes()    */
    SPIN_EHIP = 4        /* a launch failed; spin_last_hip_error() holds the runtime's message        */
} spin_status;

/* The `path` argument of the matmul calls.  It is passed as an int so that a value outside the
 * enumeration is refused with SPIN_EINVAL instead of being undefined behaviour on the library's side. */
typedef enum {
    SPIN_GEMM_LIMB_MFMA = 0, /* exact 8-bit-limb decomposition on int8 MFMA, int32 accumulation */
    SPIN_GEMM_VALU = 1       /* 64-bit multiply-add on the vector ALU (baseline)                */
} spin_gemm_path;

typedef void *spin_stream; /* hipStream_t */

/* Synthetic randomness.  The paper's parties draw masks and triples in an
 * OT-based offline phase (Section 4.2); here a stateless counter generator
 * stands in:  mix(z) is the SplitMix64 finaliser, absorb(h,v) =
 * mix(h + (v+1)*0x9E3779B97F4A7C15), and
 *   rand64(seed, stream_id, party, idx) =
 *       absorb(absorb(absorb(absorb(0, seed), stream_id), party), idx).
 * out[k] = rand64(seed, stream_id, party, first_idx + k), k < count.          */
spin_status spin_random(uint64_t *out, size_t count, uint64_t seed, uint64_t stream_id,
                        uint64_t party, uint64_t first_idx, spin_stream stream);

/* n-out-of-n arithmetic sharing (Section 4.1): x = sum_i x_i.
 * shares[i][k] = rand64(seed, stream_id, i, k) for i >= 1 and
 * shares[0][k] = x[k] - sum_{i>=1} shares[i][k].
 * x: [count] in; shares: [n][count] out.                                      */
spin_status spin_share(const uint64_t *x, size_t count, int n, uint64_t seed, uint64_t stream_id,
                       uint64_t *shares, spin_stream stream);

/* Opening (Section 4.1 reconstruction; with a mask, the E = X - A opening of
 * Section 4.3 Multiplication): out[k] = sum_i (shares[i][k] - mask[i][k]).
 * The network exchange of the paper is a reduction over the party axis here.
 * shares, mask: [n][count] in (mask may be NULL = zeros); out: [count].       */
spin_status spin_open(const uint64_t *shares, const uint64_t *mask, size_t count, int n,
                      uint64_t *out, spin_stream stream);

/* Online phase of matrix multiplication with a matrix Beaver triple
 * (Section 4.3 Multiplication; batched as in Section 7.4).  For every batch
 * entry: E = sum_i (X_i - A_i), F = sum_i (Y_i - B_i), then
 *     Z_i = C_i + E.B_i + A_i.F   and party 0 adds E.F once.
 * Row-major operands: X, A [n][batch][M][K]; Y, B [n][batch][K][N];
 * C, Z [n][batch][M][N].  Z may alias C.  For a right operand that is stored
 * transposed (Q.K^T) see spin_beaver_matmul_nt.
 * workspace: device scratch of at least
 * spin_beaver_matmul_workspace_bytes(n,batch,M,N,K,path) bytes, 256-byte
 * aligned; its contents are overwritten.  Any K is accepted: the limb path
 * splits the inner dimension so that no int32 partial sum can overflow.       */
spin_status spin_beaver_matmul(int n, int batch, int M, int N, int K,
                               const uint64_t *X, const uint64_t *Y,
                               const uint64_t *A, const uint64_t *B, const uint64_t *C,
                               uint64_t *Z, int path,
                               void *workspace, size_t workspace_bytes, spin_stream stream);

/* The same with the right operands stored transposed, the layout of K in the attention product
 * Q.K^T (Section 7.4 multiplies such pairs head by head): Yt, Bt are [n][batch][N][K] row-major and
 * Z = X . Yt^T.  Everything else, including the workspace size, as for spin_beaver_matmul; the
 * transposition costs no pass over memory (the right-hand fragments are read along rows).       */
spin_status spin_beaver_matmul_nt(int n, int batch, int M, int N, int K,
                                  const uint64_t *X, const uint64_t *Yt,
                                  const uint64_t *A, const uint64_t *Bt, const uint64_t *C,
                                  uint64_t *Z, int path,
                                  void *workspace, size_t workspace_bytes, spin_stream stream);

/* An array of Beaver matmuls of different shapes in one call (Section 7.4's PMatMul takes arrays of
 * matrices and multiplies them in parallel; products of one shape go into the batch dimension of a group,
 * different shapes into different groups).  desc: HOST array of `groups` descriptors, read before the call
 * returns; every group is what spin_beaver_matmul (y_transposed == 0) or spin_beaver_matmul_nt (!= 0) would
 * be given, with the common party count n.  On the limb path the groups share launches -- the operand packs
 * of all groups first, then their GEMMs, a handful of launches whatever the number of groups -- and every
 * group has its own part of the workspace, so the workspace must hold the SUM of the groups' needs
 * (the baseline path enqueues the groups one after another and needs the largest):
 * spin_beaver_matmul_grouped_workspace_bytes(n, groups, desc, path), 0 if a descriptor is invalid.  All
 * descriptors are validated before the first launch.  The Z of different groups must not overlap (their
 * GEMMs run concurrently).  1 <= groups <= SPIN_MAX_GROUPS.                                       */
#define SPIN_MAX_GROUPS 64
typedef struct {
    int batch, M, N, K;
    const uint64_t *X, *Y, *A, *B, *C;
    uint64_t *Z;
    int y_transposed;
} spin_matmul_group;
spin_status spin_beaver_matmul_grouped(int n, int groups, const spin_matmul_group *desc, int path,
                                       void *workspace, size_t workspace_bytes, spin_stream stream);
size_t spin_beaver_matmul_grouped_workspace_bytes(int n, int groups, const spin_matmul_group *desc,
                                                  int path);

/* Bytes of workspace spin_beaver_matmul needs; 0 if the arguments are invalid. */
size_t spin_beaver_matmul_workspace_bytes(int n, int batch, int M, int N, int K, int path);

/* spin_beaver_matmul for callers that cannot allocate device memory, and so cannot bring a workspace:
 * code running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * operands, result and checks as spin_beaver_matmul; the workspace is an array of
 * SPIN_STATIC_WORKSPACE_BYTES inside the library's device image (each GPU the library runs on holds its
 * copy until the process ends).  The call allocates and frees nothing -- no device or host memory, no
 * event objects (per-kernel timing is not recorded for it) -- and only enqueues kernels on `stream`.
 * Returns SPIN_EWORKSPACE, before anything is launched, when
 * spin_beaver_matmul_workspace_bytes(n, batch, M, N, K, path) exceeds SPIN_STATIC_WORKSPACE_BYTES.
 * All calls on one GPU share that GPU's array: two calls whose kernels may overlap in time (different
 * streams, or two replays of graphs that contain it) race and give wrong results; calls on one stream,
 * one after another, are safe.  The first call on a device looks the array's address up.          */
#define SPIN_STATIC_WORKSPACE_BYTES (64u << 20)
spin_status spin_beaver_matmul_static(int n, int batch, int M, int N, int K,
                                      const uint64_t *X, const uint64_t *Y,
                                      const uint64_t *A, const uint64_t *B, const uint64_t *C,
                                      uint64_t *Z, int path, spin_stream stream);

/* Online phase of elementwise multiplication with scalar triples (Section 4.3;
 * the "batch multiplication" of Section 7.3):
 *     e = sum_i (x_i - a_i), f = sum_i (y_i - b_i),
 *     z_i = c_i + e*b_i + a_i*f  (+ e*f for i = 0).
 * x, y, a, b, c: [n][count] in; z: [n][count] out; z may alias any input.     */
spin_status spin_beaver_mul(int n, size_t count,
                            const uint64_t *x, const uint64_t *y,
                            const uint64_t *a, const uint64_t *b, const uint64_t *c,
                            uint64_t *z, spin_stream stream);

/* The same with one factor tiled, the batch multiplication E * R of Section 7.3 in which the smaller
 * array is repeated along one axis up to the size of the other (and its downsized form R * V).  The
 * large operands y, b, c and the result z are [n][outer][mid][inner]; the small factor x and its mask a
 * are [n][outer][mid] when over_inner != 0 (one factor per row, repeated along inner) and
 * [n][outer][inner] when over_inner == 0 (one factor per column, repeated along mid).  With xt, at the
 * tiled arrays, z equals spin_beaver_mul(n, outer*mid*inner, xt, y, at, b, c); the triple satisfies
 * sum_i c_i = (tiled sum_i a_i) * (sum_i b_i).  The tiled arrays are never formed: 4n instead of 6n
 * words move per element.  z may alias y, b or c.                                                   */
spin_status spin_beaver_mul_bcast(int n, size_t outer, size_t mid, size_t inner, int over_inner,
                                  const uint64_t *x, const uint64_t *y,
                                  const uint64_t *a, const uint64_t *b, const uint64_t *c,
                                  uint64_t *z, spin_stream stream);

/* Signed probabilistic truncation by f bits (Section 4.4 Truncation):
 * Truncate(x,f) = UnsignedTruncate(x + 2^62, 64, f) - 2^(62-f), correct up to
 * one unit for x in [-2^62, 2^62-1] and undefined (not an error) outside.
 * The dealer tuple per element is a random ring element r with sharings of r,
 * of r_top = bits f..62 of r and of r_msb = bit 63 of r.  Steps:
 *     c = sum_i (x_i + r_i) + 2^62;  c_msb = c >> 63;  c' = bits f..62 of c;
 *     b_i   = r_msb_i + [i=0] c_msb - 2 c_msb r_msb_i;
 *     out_i = [i=0] c' - r_top_i + 2^(63-f) b_i - [i=0] 2^(62-f).
 * x, r, r_top, r_msb: [n][count] in; out: [n][count], may alias x.
 * 1 <= f <= 61.                                                               */
spin_status spin_trunc(int n, size_t count, int f, const uint64_t *x,
                       const uint64_t *r, const uint64_t *r_top, const uint64_t *r_msb,
                       uint64_t *out, spin_stream stream);

/* Fixed-point multiplication in one pass: spin_beaver_mul followed by spin_trunc of its result
 * (a product carries twice the precision, Section 4.3; Truncate brings it back, Section 4.4), with
 * the product shares kept in registers instead of written and read again.  out equals
 * spin_trunc(n, count, f, z, r, r_top, r_msb) of z = spin_beaver_mul(n, count, x, y, a, b, c) word
 * for word.  Shapes and aliasing as for those two calls; out may alias any input.  1 <= f <= 61. */
spin_status spin_beaver_mul_trunc(int n, size_t count, int f,
                                  const uint64_t *x, const uint64_t *y,
                                  const uint64_t *a, const uint64_t *b, const uint64_t *c,
                                  const uint64_t *r, const uint64_t *r_top, const uint64_t *r_msb,
                                  uint64_t *out, spin_stream stream);

/* Public-coefficient linear combination followed by one truncation: the local
 * part of Scale and Add (Section 4.3) and the single deferred truncation of
 * polynomial evaluation (Section 4.4, Polynomial evaluation; the fused
 * (p+6)-bit truncation of Section 7.2, Eq. (4)):
 *     y_i   = sum_j coef[j] * in[j]_i  +  [i=0] constant          (local)
 *     out   = f > 0 ? Truncate(y, f) : y                           (as spin_trunc)
 * in:   HOST array of `terms` DEVICE pointers, each a [n][count] share tensor;
 * coef: HOST array of `terms` public ring coefficients; 1 <= terms <= SPIN_MAX_TERMS.
 * r, r_top, r_msb: truncation tuple as in spin_trunc (ignored, may be NULL,
 * when f = 0).  out: [n][count], may alias any input.  0 <= f <= 61.          */
#define SPIN_MAX_TERMS 8
spin_status spin_lincomb_trunc(int n, size_t count, int terms, const uint64_t *const *in,
                               const uint64_t *coef, uint64_t constant, int f,
                               const uint64_t *r, const uint64_t *r_top, const uint64_t *r_msb,
                               uint64_t *out, spin_stream stream);

/* Binary sharing (Section 4.1): 64 independent bit positions per word,
 * x = XOR_i x_i.  XOR of sharings is local (Section 4.3 Addition); AND consumes
 * a bit triple (a, b, c = a AND b) and is the GF(2) form of the Beaver update.
 *   spin_bshare:     shares[i][k] = rand64(seed, stream_id, i, k) for i >= 1,
 *                    shares[0][k] = x[k] XOR (XOR of the others).
 *   spin_bopen:      out[k] = XOR_i (shares[i][k] XOR mask[i][k]); mask may be NULL.
 *   spin_beaver_and: e = XOR_i (x_i ^ a_i), f = XOR_i (y_i ^ b_i),
 *                    z_i = c_i ^ (e & b_i) ^ (a_i & f)  (^ (e & f) for i = 0).
 * Layouts as for the arithmetic calls: [n][count] words; z may alias an input. */
spin_status spin_bshare(const uint64_t *x, size_t count, int n, uint64_t seed, uint64_t stream_id,
                        uint64_t *shares, spin_stream stream);
spin_status spin_bopen(const uint64_t *shares, const uint64_t *mask, size_t count, int n,
                       uint64_t *out, spin_stream stream);
spin_status spin_beaver_and(int n, size_t count,
                            const uint64_t *x, const uint64_t *y,
                            const uint64_t *a, const uint64_t *b, const uint64_t *c,
                            uint64_t *z, spin_stream stream);

/* The same calls over the ring Z_2^128 (the paper's second ring width, Section 6: "64-bit or
 * 128-bit"; its own kernels multiply __int128, Section 6.1).  A ring element is 16 bytes,
 * little-endian: two uint64_t words, low word first (the layout of unsigned __int128).  Pointers
 * are passed as uint64_t* to those words; `count` and the matrix dimensions count ring elements;
 * tensors are party-major as before.  A 128-bit generator word is the pair of 64-bit generator
 * outputs at indices 2k (low) and 2k+1 (high).  spin128_trunc: Truncate(x,f) =
 * UnsignedTruncate(x + 2^126, 128, f) - 2^(126-f), tuple fields r_top = bits f..126 and
 * r_msb = bit 127 of r, 1 <= f <= 125.  Everything else as documented at the 64-bit call.       */
spin_status spin128_share(const uint64_t *x, size_t count, int n, uint64_t seed, uint64_t stream_id,
                          uint64_t *shares, spin_stream stream);
spin_status spin128_open(const uint64_t *shares, const uint64_t *mask, size_t count, int n,
                         uint64_t *out, spin_stream stream);
spin_status spin128_beaver_matmul(int n, int batch, int M, int N, int K,
                                  const uint64_t *X, const uint64_t *Y,
                                  const uint64_t *A, const uint64_t *B, const uint64_t *C,
                                  uint64_t *Z, int path,
                                  void *workspace, size_t workspace_bytes, spin_stream stream);
size_t spin128_beaver_matmul_workspace_bytes(int n, int batch, int M, int N, int K, int path);
spin_status spin128_beaver_mul(int n, size_t count,
                               const uint64_t *x, const uint64_t *y,
                               const uint64_t *a, const uint64_t *b, const uint64_t *c,
                               uint64_t *z, spin_stream stream);
spin_status spin128_trunc(int n, size_t count, int f, const uint64_t *x,
                          const uint64_t *r, const uint64_t *r_top, const uint64_t *r_msb,
                          uint64_t *out, spin_stream stream);

/* The same calls over the ring Z_2^32, the Fixed32 representation of Section 7.1 (mixing bit
 * lengths): steps that do not need 64 bits run on 32-bit shares at half the bytes.  Ring elements
 * are uint32_t, tensors party-major as before.  A 32-bit generator word is the low half of
 * rand64 at the same index.  spin32_trunc: Truncate(x,f) = UnsignedTruncate(x + 2^30, 32, f) -
 * 2^(30-f), tuple fields r_top = bits f..30 and r_msb = bit 31 of r, 1 <= f <= 29.  The limb
 * path of spin32_beaver_matmul uses four digits (10 digit pairs) and never splits the inner
 * dimension.  Everything else as documented at the 64-bit call.
 *
 * spin_cast_64_to_32 is the local Fixed64 -> Fixed32 cast of Section 7.1: out[k] = low 32 bits
 * of in[k], applied by every party to its own share (pass all n*count share words at once);
 * the opened value is preserved while it lies in [-2^31, 2^31).  in: [count] uint64_t,
 * out: [count] uint32_t, must not overlap.                                                      */
spin_status spin32_share(const uint32_t *x, size_t count, int n, uint64_t seed, uint64_t stream_id,
                         uint32_t *shares, spin_stream stream);
spin_status spin32_open(const uint32_t *shares, const uint32_t *mask, size_t count, int n,
                        uint32_t *out, spin_stream stream);
spin_status spin32_beaver_matmul(int n, int batch, int M, int N, int K,
                                 const uint32_t *X, const uint32_t *Y,
                                 const uint32_t *A, const uint32_t *B, const uint32_t *C,
                                 uint32_t *Z, int path,
                                 void *workspace, size_t workspace_bytes, spin_stream stream);
size_t spin32_beaver_matmul_workspace_bytes(int n, int batch, int M, int N, int K, int path);
spin_status spin32_beaver_mul(int n, size_t count,
                              const uint32_t *x, const uint32_t *y,
                              const uint32_t *a, const uint32_t *b, const uint32_t *c,
                              uint32_t *z, spin_stream stream);
spin_status spin32_trunc(int n, size_t count, int f, const uint32_t *x,
                         const uint32_t *r, const uint32_t *r_top, const uint32_t *r_msb,
                         uint32_t *out, spin_stream stream);
spin_status spin_cast_64_to_32(const uint64_t *in, size_t count, uint32_t *out, spin_stream stream);

/* Static description of a status code. */
const char *spin_status_string(int status);

/* Message of the most recent HIP failure seen by this thread ("" if none). */
const char *spin_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SPIN_H */
