/* Host-side sanitizer target for the C ABI's argument checks: the library's entry-point source (spin_api.hip, host
 * code) is compiled with -fsanitize=address,undefined and linked into this program, which calls every exported
 * function with the arguments that must be refused -- null, misaligned, out-of-range sizes, missing workspace, bad
 * descriptor arrays -- and checks the status codes.  Validation happens before any launch and touches no HIP call,
 * so the program runs on a machine without a GPU; pointers that pass validation are never handed over here.
 * Built and run by tests/test_sanitizers.py. */
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "spin.h"
#include "spin_bench.h"

static int failures = 0;
#define EXPECT(call, want) do { spin_status got_ = (call); if (got_ != (want)) { \
    printf("FAILED line %d: %s -> %d (%s), wanted %d\n", __LINE__, #call, (int)got_, spin_status_string(got_), (int)(want)); ++failures; } } while (0)

int main(void)
{
    uint64_t *ok = (uint64_t *)(uintptr_t)0x10000;      /* aligned, never dereferenced: every call below is refused first */
    uint64_t *odd = (uint64_t *)(uintptr_t)0x10008;
    uint32_t *ok32 = (uint32_t *)(uintptr_t)0x10000;
    const size_t huge = (size_t)1 << 40;

    EXPECT(spin_random(NULL, 8, 1, 1, 1, 0, NULL), SPIN_EINVAL);
    EXPECT(spin_random(ok, 0, 1, 1, 1, 0, NULL), SPIN_EINVAL);
    EXPECT(spin_random(ok, huge, 1, 1, 1, 0, NULL), SPIN_ERANGE);
    EXPECT(spin_share(NULL, 8, 2, 1, 1, ok, NULL), SPIN_EINVAL);
    EXPECT(spin_share(ok, 8, 0, 1, 1, ok, NULL), SPIN_EINVAL);
    EXPECT(spin_share(ok, 8, SPIN_MAX_PARTIES + 1, 1, 1, ok, NULL), SPIN_EINVAL);
    EXPECT(spin_share(odd, 8, 2, 1, 1, ok, NULL), SPIN_EINVAL);
    EXPECT(spin_share(ok, huge, 2, 1, 1, ok, NULL), SPIN_ERANGE);
    EXPECT(spin_open(ok, odd, 8, 2, ok, NULL), SPIN_EINVAL);
    EXPECT(spin_open(ok, NULL, 8, 9, ok, NULL), SPIN_EINVAL);
    EXPECT(spin_open(ok, NULL, huge, 2, ok, NULL), SPIN_ERANGE);
    EXPECT(spin_beaver_mul(2, 8, ok, ok, ok, ok, NULL, ok, NULL), SPIN_EINVAL);
    EXPECT(spin_beaver_mul(2, 0, ok, ok, ok, ok, ok, ok, NULL), SPIN_EINVAL);
    EXPECT(spin_beaver_mul(2, huge, ok, ok, ok, ok, ok, ok, NULL), SPIN_ERANGE);
    EXPECT(spin_beaver_mul_trunc(2, 8, 0, ok, ok, ok, ok, ok, ok, ok, ok, ok, NULL), SPIN_EINVAL);
    EXPECT(spin_beaver_mul_trunc(2, 8, 16, ok, ok, ok, ok, ok, ok, NULL, ok, ok, NULL), SPIN_EINVAL);
    EXPECT(spin_beaver_mul_bcast(2, 0, 4, 4, 1, ok, ok, ok, ok, ok, ok, NULL), SPIN_EINVAL);
    EXPECT(spin_beaver_mul_bcast(2, huge, huge, 4, 1, ok, ok, ok, ok, ok, ok, NULL), SPIN_ERANGE);
    EXPECT(spin_trunc(2, 8, 0, ok, ok, ok, ok, ok, NULL), SPIN_EINVAL);
    EXPECT(spin_trunc(2, 8, 62, ok, ok, ok, ok, ok, NULL), SPIN_EINVAL);
    EXPECT(spin_trunc(2, 8, 16, ok, ok, ok, NULL, ok, NULL), SPIN_EINVAL);

    EXPECT(spin_beaver_matmul(2, 1, 0, 4, 4, ok, ok, ok, ok, ok, ok, SPIN_GEMM_LIMB_MFMA, ok, 1 << 30, NULL), SPIN_EINVAL);
    EXPECT(spin_beaver_matmul(2, 1, 4, 4, 4, ok, ok, ok, ok, ok, ok, 7, ok, 1 << 30, NULL), SPIN_EINVAL);
    EXPECT(spin_beaver_matmul(2, 1, 4, 4, 4, ok, odd, ok, ok, ok, ok, SPIN_GEMM_VALU, ok, 1 << 30, NULL), SPIN_EINVAL);
    EXPECT(spin_beaver_matmul(2, 1, 4, 4, 4, ok, ok, ok, ok, ok, ok, SPIN_GEMM_LIMB_MFMA, NULL, 1 << 30, NULL), SPIN_EWORKSPACE);
    EXPECT(spin_beaver_matmul(2, 1, 4, 4, 4, ok, ok, ok, ok, ok, ok, SPIN_GEMM_LIMB_MFMA, ok, 16, NULL), SPIN_EWORKSPACE);
    EXPECT(spin_beaver_matmul(2, 1, 4, 4, 4, ok, ok, ok, ok, ok, ok, SPIN_GEMM_LIMB_MFMA, (void *)(uintptr_t)0x10010, 1 << 30, NULL), SPIN_EWORKSPACE);
    EXPECT(spin_beaver_matmul(2, 1, 1 << 25, 4, 4, ok, ok, ok, ok, ok, ok, SPIN_GEMM_LIMB_MFMA, ok, 1 << 30, NULL), SPIN_ERANGE);
    EXPECT(spin_beaver_matmul(8, 60000, 4, 4, 4, ok, ok, ok, ok, ok, ok, SPIN_GEMM_LIMB_MFMA, ok, 1 << 30, NULL), SPIN_ERANGE);
    EXPECT(spin_beaver_matmul_nt(2, 1, 4, 0, 4, ok, ok, ok, ok, ok, ok, SPIN_GEMM_LIMB_MFMA, ok, 1 << 30, NULL), SPIN_EINVAL);
    EXPECT(spin_beaver_matmul_static(2, 1, 2048, 2048, 2048, ok, ok, ok, ok, ok, ok, SPIN_GEMM_LIMB_MFMA, NULL), SPIN_EWORKSPACE);
    EXPECT(spin_beaver_matmul_static(2, 1, 8, 8, 8, ok, ok, NULL, ok, ok, ok, SPIN_GEMM_LIMB_MFMA, NULL), SPIN_EINVAL);
    if (spin_beaver_matmul_workspace_bytes(2, 1, 0, 4, 4, SPIN_GEMM_LIMB_MFMA) != 0) { printf("FAILED: workspace of an invalid shape\n"); ++failures; }
    if (spin_beaver_matmul_workspace_bytes(5, 1, 4096, 4096, 4096, SPIN_GEMM_LIMB_MFMA) == 0) { printf("FAILED: workspace of config 5\n"); ++failures; }
    if (spin128_beaver_matmul_workspace_bytes(2, 1, 100, 100, 100, SPIN_GEMM_VALU) == 0) { printf("FAILED: workspace 128\n"); ++failures; }
    if (spin32_beaver_matmul_workspace_bytes(2, 1, 100, 100, 100, 9) != 0) { printf("FAILED: workspace 32, bad path\n"); ++failures; }

    {   /* grouped call: descriptor arrays of every admissible and inadmissible length */
        spin_matmul_group desc[SPIN_MAX_GROUPS];
        for (int g = 0; g < SPIN_MAX_GROUPS; ++g) {
            spin_matmul_group d = {1 + g % 3, 8 + g, 8, 8 + 2 * g, ok, ok, ok, ok, ok, ok, g % 2};
            desc[g] = d;
        }
        if (spin_beaver_matmul_grouped_workspace_bytes(3, SPIN_MAX_GROUPS, desc, SPIN_GEMM_LIMB_MFMA) == 0) { printf("FAILED: grouped workspace\n"); ++failures; }
        EXPECT(spin_beaver_matmul_grouped(3, 0, desc, SPIN_GEMM_LIMB_MFMA, ok, 1 << 30, NULL), SPIN_EINVAL);
        EXPECT(spin_beaver_matmul_grouped(3, SPIN_MAX_GROUPS + 1, desc, SPIN_GEMM_LIMB_MFMA, ok, 1 << 30, NULL), SPIN_EINVAL);
        EXPECT(spin_beaver_matmul_grouped(3, SPIN_MAX_GROUPS, NULL, SPIN_GEMM_LIMB_MFMA, ok, 1 << 30, NULL), SPIN_EINVAL);
        EXPECT(spin_beaver_matmul_grouped(3, SPIN_MAX_GROUPS, desc, SPIN_GEMM_LIMB_MFMA, ok, 64, NULL), SPIN_EWORKSPACE);
        desc[SPIN_MAX_GROUPS - 1].K = 0;
        EXPECT(spin_beaver_matmul_grouped(3, SPIN_MAX_GROUPS, desc, SPIN_GEMM_LIMB_MFMA, ok, 1 << 30, NULL), SPIN_EINVAL);
        desc[SPIN_MAX_GROUPS - 1].K = 8;
        desc[5].Z = NULL;
        EXPECT(spin_beaver_matmul_grouped(3, SPIN_MAX_GROUPS, desc, SPIN_GEMM_VALU, ok, 1 << 30, NULL), SPIN_EINVAL);
    }
    {   /* linear combination: host arrays of pointers and coefficients of every length */
        const uint64_t *in[SPIN_MAX_TERMS + 1];
        uint64_t coef[SPIN_MAX_TERMS + 1];
        for (int j = 0; j <= SPIN_MAX_TERMS; ++j) { in[j] = ok; coef[j] = 3 + j; }
        EXPECT(spin_lincomb_trunc(2, 8, 0, in, coef, 0, 0, NULL, NULL, NULL, ok, NULL), SPIN_EINVAL);
        EXPECT(spin_lincomb_trunc(2, 8, SPIN_MAX_TERMS + 1, in, coef, 0, 0, NULL, NULL, NULL, ok, NULL), SPIN_EINVAL);
        EXPECT(spin_lincomb_trunc(2, 8, SPIN_MAX_TERMS, in, coef, 0, 16, ok, NULL, ok, ok, NULL), SPIN_EINVAL);
        EXPECT(spin_lincomb_trunc(2, 8, SPIN_MAX_TERMS, NULL, coef, 0, 0, NULL, NULL, NULL, ok, NULL), SPIN_EINVAL);
        in[SPIN_MAX_TERMS - 1] = odd;
        EXPECT(spin_lincomb_trunc(2, 8, SPIN_MAX_TERMS, in, coef, 0, 0, NULL, NULL, NULL, ok, NULL), SPIN_EINVAL);
        EXPECT(spin_lincomb_trunc(2, huge, 1, in, coef, 0, 0, NULL, NULL, NULL, ok, NULL), SPIN_ERANGE);
    }
    EXPECT(spin_bshare(ok, 8, 9, 1, 1, ok, NULL), SPIN_EINVAL);
    EXPECT(spin_bopen(NULL, NULL, 8, 2, ok, NULL), SPIN_EINVAL);
    EXPECT(spin_beaver_and(2, 8, ok, ok, ok, odd, ok, ok, NULL), SPIN_EINVAL);
    EXPECT(spin128_share(ok, huge, 2, 1, 1, ok, NULL), SPIN_ERANGE);
    EXPECT(spin128_open(ok, NULL, 8, 0, ok, NULL), SPIN_EINVAL);
    EXPECT(spin128_beaver_matmul(2, 1, 4, 4, 4, ok, ok, ok, ok, ok, ok, SPIN_GEMM_LIMB_MFMA, ok, 16, NULL), SPIN_EWORKSPACE);
    EXPECT(spin128_beaver_mul(2, 8, ok, NULL, ok, ok, ok, ok, NULL), SPIN_EINVAL);
    EXPECT(spin128_trunc(2, 8, 126, ok, ok, ok, ok, ok, NULL), SPIN_EINVAL);
    EXPECT(spin32_share(ok32, 8, 0, 1, 1, ok32, NULL), SPIN_EINVAL);
    EXPECT(spin32_open(ok32, NULL, 0, 2, ok32, NULL), SPIN_EINVAL);
    EXPECT(spin32_beaver_matmul(2, 1, 4, 4, 4, ok32, ok32, ok32, ok32, ok32, ok32, SPIN_GEMM_LIMB_MFMA, NULL, 0, NULL), SPIN_EWORKSPACE);
    EXPECT(spin32_beaver_mul(2, 8, ok32, ok32, ok32, ok32, ok32, NULL, NULL), SPIN_EINVAL);
    EXPECT(spin32_trunc(2, 8, 30, ok32, ok32, ok32, ok32, ok32, NULL), SPIN_EINVAL);
    EXPECT(spin_cast_64_to_32(ok, 0, ok32, NULL), SPIN_EINVAL);
    EXPECT(spin_probe_mfma(ok, 0, 10, ok, NULL), SPIN_EINVAL);
    {
        double ms = 0.0; unsigned cnt = 0;
        EXPECT(spin_profile_read(99, &ms, &cnt), SPIN_EINVAL);
        EXPECT(spin_profile_read(SPIN_KERNEL_SHARE, NULL, &cnt), SPIN_EINVAL);
        EXPECT(spin_profile_read(SPIN_KERNEL_SHARE, &ms, &cnt), SPIN_OK);      /* nothing recorded: zero launches */
        if (cnt != 0) { printf("FAILED: launches recorded\n"); ++failures; }
        spin_profile_reset();
    }
    for (int st = 0; st <= 5; ++st)
        if (strlen(spin_status_string(st)) == 0) { printf("FAILED: empty status string\n"); ++failures; }
    if (spin_last_hip_error() == NULL) { printf("FAILED: last error string\n"); ++failures; }
    if (failures) { printf("%d check(s) failed\n", failures); return 1; }
    printf("abi sanitizer run ok\n");
    return 0;
}
