// Drives every C-ABI entry point through its validation paths (bad and good arguments; the launchers are
// stubs); built with host sanitizers by tests/test_sanitizers_host.py, which checks the exit status and
// the statuses printed here.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "../../include/fa_mi355.h"

static int failures = 0;
#define EXPECT(call, want)                                                         \
    do {                                                                           \
        int got = (call);                                                          \
        if (got != (want)) {                                                       \
            printf("line %d: %s = %d (%s), wanted %d\n", __LINE__, #call, got, fa_status_string(got), want); \
            ++failures;                                                            \
        }                                                                          \
    } while (0)

int main() {
    void* p = aligned_alloc(256, 4096);
    void* odd = (char*)p + 8;
    float* f = (float*)p;
    for (int st = -1; st <= 9; ++st)
        if (!fa_status_string(st) || !fa_status_string(st)[0]) ++failures;
    // forward
    EXPECT(fa_fwd(p, p, p, p, f, 1, 2, 16, 128, 0.1f, 0, FA_BF16, 0), FA_OK);
    EXPECT(fa_fwd(0, p, p, p, f, 1, 2, 16, 128, 0.1f, 0, FA_BF16, 0), FA_ERR_NULL);
    EXPECT(fa_fwd(p, p, p, p, f, 1, 2, 16, 128, 0.1f, 0, 7, 0), FA_ERR_DTYPE);
    EXPECT(fa_fwd(p, p, p, p, f, 0, 2, 16, 128, 0.1f, 0, FA_BF16, 0), FA_ERR_SHAPE);
    EXPECT(fa_fwd(p, p, p, p, f, 1, 2, 16, 128, NAN, 0, FA_BF16, 0), FA_ERR_SHAPE);
    EXPECT(fa_fwd(p, p, p, p, f, 1, 2, 16, 128, 0.1f, 2, FA_BF16, 0), FA_ERR_SHAPE);
    EXPECT(fa_fwd(p, p, p, p, f, 1, 2, 16, 96, 0.1f, 0, FA_BF16, 0), FA_ERR_UNSUPPORTED);
    EXPECT(fa_fwd(p, odd, p, p, f, 1, 2, 16, 128, 0.1f, 0, FA_BF16, 0), FA_ERR_ALIGN);
    EXPECT(fa_fwd(p, p, p, p, f, 65536, 65536, 16, 128, 0.1f, 0, FA_BF16, 0), FA_ERR_SHAPE);
    EXPECT(fa_fwd(p, p, p, p, f, 1, 1, 0x7ff00000 / 512 + 1, 128, 0.1f, 0, FA_BF16, 0), FA_ERR_UNSUPPORTED);
    EXPECT(fa_fwd_schedule(p, p, p, p, f, 1, 2, 16, 128, 0.1f, 0, FA_F16, FA_SCHED_PINGPONG, 0), FA_OK);
    EXPECT(fa_fwd_schedule(p, p, p, p, f, 1, 2, 16, 128, 0.1f, 0, FA_F16, 9, 0), FA_ERR_SHAPE);
    EXPECT(fa_fwd_schedule(p, p, p, p, f, 1, 2, 16, 128, 0.1f, 0, FA_F32, FA_SCHED_PINGPONG, 0), FA_ERR_UNSUPPORTED);
    EXPECT(fa_fwd_gqa(p, p, p, p, f, 1, 6, 4, 16, 128, 0.1f, 0, FA_BF16, 0), FA_ERR_SHAPE);
    EXPECT(fa_fwd_gqa(p, p, p, p, f, 1, 6, 3, 16, 128, 0.1f, 0, FA_BF16, 0), FA_OK);
    // FP8
    EXPECT(fa_fwd_fp8(p, p, p, f, f, f, p, f, 1, 2, 16, 128, 128, 0.1f, 1, 0), FA_OK);
    EXPECT(fa_fwd_fp8(p, p, p, f, 0, f, p, f, 1, 2, 16, 128, 128, 0.1f, 1, 0), FA_ERR_NULL);
    EXPECT(fa_fwd_fp8(p, p, p, f, f, f, p, f, 1, 2, 16, 128, 64, 0.1f, 1, 0), FA_ERR_UNSUPPORTED);
    EXPECT(fa_fwd_fp8_gqa(p, p, p, f, f, f, p, f, 1, 4, 0, 16, 128, 128, 0.1f, 1, 0), FA_ERR_SHAPE);
    EXPECT(fa_fp8_quant_hadamard(p, FA_BF16, p, f, 1, 2, 16, 128, 128, 0, 0, 0), FA_OK);
    EXPECT(fa_fp8_quant_hadamard(p, FA_FP8_E4M3, p, f, 1, 2, 16, 128, 128, 0, 0, 0), FA_ERR_UNSUPPORTED);
    EXPECT(fa_fp8_quant_hadamard(p, FA_BF16, p, f, 1, 2, 16, 128, 128, 0, 3, 0), FA_ERR_SHAPE);
    EXPECT(fa_fp8_quant_hadamard(p, -1, p, f, 1, 2, 16, 128, 128, 0, 0, 0), FA_ERR_DTYPE);
    // backward
    const size_t ws = fa_bwd_workspace_bytes(1, 2, 16, 128, FA_BF16);
    if (ws != 128 || fa_bwd_workspace_bytes(1, 2, 16, 96, FA_BF16) != 0) ++failures;
    EXPECT(fa_bwd(p, p, p, p, f, p, p, p, p, p, ws, 1, 2, 16, 128, 0.1f, 0, FA_BF16, 0), FA_OK);
    EXPECT(fa_bwd(p, p, p, p, f, p, p, p, p, p, ws - 1, 1, 2, 16, 128, 0.1f, 0, FA_BF16, 0), FA_ERR_WORKSPACE);
    EXPECT(fa_bwd(p, p, p, p, f, p, p, p, p, 0, ws, 1, 2, 16, 128, 0.1f, 0, FA_BF16, 0), FA_ERR_WORKSPACE);
    EXPECT(fa_bwd(p, p, p, p, f, p, p, p, p, odd, ws, 1, 2, 16, 128, 0.1f, 0, FA_BF16, 0), FA_ERR_ALIGN);
    EXPECT(fa_bwd(p, p, p, p, f, p, p, p, p, p, ws, 1, 2, 16, 128, 0.1f, 0, FA_F32, 0), FA_ERR_UNSUPPORTED);
    EXPECT(fa_bwd_gqa(p, p, p, p, f, p, p, p, p, p, ws, 1, 2, 1, 16, 128, 0.1f, 0, FA_F16, 0), FA_OK);
    EXPECT(fa_bwd_noalloc(p, p, p, p, f, p, p, p, p, 4, 1, FA_BWD_NOALLOC_MAX_ROWS / 4 + 1, 64, 0.1f, 0, FA_BF16, 0),
           FA_ERR_TOO_LARGE);
    EXPECT(fa_bwd_noalloc(p, p, p, 0, f, p, p, p, p, 1, 2, 16, 128, 0.1f, 0, FA_BF16, 0), FA_ERR_NULL);
    // introspection and the probe
    if (fa_fwd_kernel_name(FA_BF16, 16, 96, 0) != 0 || fa_fwd_kernel_name(FA_BF16, 16, 128, 0) == 0) ++failures;
    if (fa_probe_mfma_flops(FA_F16, 10) != 0.0) ++failures;
    EXPECT(fa_probe_mfma(p, 1024, f, FA_BF16, 10, 0), FA_OK);
    EXPECT(fa_probe_mfma(p, 1000, f, FA_BF16, 10, 0), FA_ERR_SHAPE);
    EXPECT(fa_probe_mfma(p, 1024, f, FA_F16, 10, 0), FA_ERR_UNSUPPORTED);
    free(p);
    printf("api sanitizer run: %d failures\n", failures);
    return failures ? 1 : 0;
}
