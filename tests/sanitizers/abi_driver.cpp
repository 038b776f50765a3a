// Sanitizer driver for the host half of the C ABI (argument checks, slice planning, workspace
// arithmetic, overlap logic).  Built by tests/test_sanitizers.py from
// paper_2505_09326_amd/csrc/sphattn_api.hip with the HOST code under
// -fsanitize=address,undefined (device code is compiled as usual and never runs here).
// Every call below must return before any launch: the pointers are fake addresses that are
// never dereferenced, or the arithmetic is host-only.  Exits non-zero on the first unexpected
// return code; the sanitizers abort on undefined behaviour or a bad access.
#include <limits.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "../../include/sphattn.h"

static int failures = 0;
#define EXPECT(call, want) do { const long long got_ = (long long)(call); if (got_ != (long long)(want)) { \
    fprintf(stderr, "%s:%d: %s = %lld, expected %lld\n", __FILE__, __LINE__, #call, got_, (long long)(want)); ++failures; } } while (0)

static void* P(uintptr_t a) { return (void*)a; }

int main()
{
    void *Q = P(0x1000000), *K = P(0x2000000), *V = P(0x3000000), *O = P(0x4000000), *W = P(0x40000000);
    // plain forward and twins: every validation branch
    EXPECT(sphattn_fwd(nullptr, K, V, O, 1, 1, 128, 128, SPHATTN_BF16, nullptr), SPHATTN_ERR_NULL);
    EXPECT(sphattn_fwd(Q, K, V, O, 0, 1, 128, 128, SPHATTN_BF16, nullptr), SPHATTN_ERR_SHAPE);
    EXPECT(sphattn_fwd(Q, K, V, O, 1, 1, INT_MAX, 128, SPHATTN_BF16, nullptr), SPHATTN_ERR_SHAPE);
    EXPECT(sphattn_fwd(Q, K, V, O, INT_MAX, INT_MAX, INT_MAX, 128, SPHATTN_F32, nullptr), SPHATTN_ERR_SHAPE);
    EXPECT(sphattn_fwd(Q, K, V, O, 1, 1, 128, 96, SPHATTN_BF16, nullptr), SPHATTN_ERR_HEAD_DIM);
    EXPECT(sphattn_fwd(Q, K, V, O, 1, 1, 128, 128, 17, nullptr), SPHATTN_ERR_DTYPE);
    EXPECT(sphattn_fwd(P(0x1000008), K, V, O, 1, 1, 128, 128, SPHATTN_BF16, nullptr), SPHATTN_ERR_ALIGN);
    EXPECT(sphattn_fwd(Q, K, V, Q, 1, 1, 128, 128, SPHATTN_BF16, nullptr), SPHATTN_ERR_ALIAS);
    EXPECT(sphattn_fwd(Q, K, V, P(UINTPTR_MAX - 4095), 1, 1, 128, 128, SPHATTN_BF16, nullptr), SPHATTN_ERR_SHAPE);   // O would wrap the address space
    EXPECT(sphattn_fwd(P(UINTPTR_MAX - 4095), K, V, O, 1, 1, 128, 128, SPHATTN_BF16, nullptr), SPHATTN_ERR_SHAPE);
    EXPECT(sphattn_fwd_tile_rows(Q, K, V, O, nullptr, 1, 1, 128, 128, SPHATTN_BF16, 64, nullptr), SPHATTN_ERR_SHAPE);
    EXPECT(sphattn_softmax_fwd(Q, K, V, O, 1, 1, 128, 128, SPHATTN_F32, nullptr), SPHATTN_ERR_DTYPE);
    EXPECT(sphattn_normalized_fwd(Q, K, V, O, 1, 1, 128, 128, SPHATTN_BF16, 9, nullptr), SPHATTN_ERR_NORMALIZER);
    EXPECT(sphattn_grn_fwd(Q, K, V, (const float*)P(0x5000002), O, 1, 4, 2, 128, 64, SPHATTN_BF16, nullptr), SPHATTN_ERR_ALIGN);
    EXPECT(sphattn_grn_fwd(Q, K, V, nullptr, O, 1, 4, 3, 128, 64, SPHATTN_BF16, nullptr), SPHATTN_ERR_SHAPE);
    EXPECT(sphattn_cross_fwd(Q, K, V, nullptr, O, (float*)O, 1, 4, 2, 100, 300, 64, SPHATTN_BF16, nullptr), SPHATTN_ERR_ALIAS);
    EXPECT(sphattn_partial_fwd(Q, K, V, nullptr, (float*)O, nullptr, 1, 4, 2, 100, 300, 64, SPHATTN_BF16, nullptr), SPHATTN_ERR_NULL);
    EXPECT(sphattn_combine((const float*)Q, (const float*)K, 0, O, nullptr, 1, 1, 64, 64, SPHATTN_BF16, nullptr), SPHATTN_ERR_SHAPE);
    EXPECT(sphattn_combine((const float*)Q, (const float*)K, 65536, Q, nullptr, 1, 1, 64, 64, SPHATTN_BF16, nullptr), SPHATTN_ERR_ALIAS);

    // slice planning: any n_splits >= 0, any N the shape check lets through
    const int counts[] = {0, 1, 2, 3, 15, 16, 17, 1000, INT_MAX - 1, INT_MAX};
    for (int n : counts) {
        const int rc = sphattn_splitkv_fwd(Q, K, V, nullptr, O, nullptr, 1, 1, 1, 1024, 128, SPHATTN_BF16, n, W, 1, nullptr);
        EXPECT(rc, SPHATTN_ERR_WORKSPACE);         // planned, then one byte of workspace is too little
    }
    EXPECT(sphattn_splitkv_fwd(Q, K, V, nullptr, O, nullptr, 1, 1, 1, 1024, 128, SPHATTN_BF16, -1, W, (size_t)1 << 40, nullptr), SPHATTN_ERR_SHAPE);
    EXPECT(sphattn_splitkv_workspace_bytes(1, 2, 1000, 128, 4), (((size_t)4 * 2000 * 129 * 4 + 255) & ~(size_t)255));
    EXPECT(sphattn_splitkv_workspace_bytes(INT_MAX, INT_MAX, INT_MAX, 128, INT_MAX), 0);
    EXPECT(sphattn_splitkv_workspace_bytes(1, 1, 1, 128, 0), 0);
    // the heuristic over a sweep of shapes, including the largest ints: always 1 .. number of tiles
    uint64_t s = 12345;
    for (int it = 0; it < 20000; ++it) {
        s = s * 6364136223846793005ULL + 1442695040888963407ULL;
        const int B = 1 + (int)((s >> 60) & 7), H = 1 + (int)((s >> 54) & 31);
        const int N = it % 50 == 0 ? INT_MAX - (int)((s >> 33) & 1023) : 1 + (int)((s >> 20) & 0xfffff);
        const int d = (s >> 8) & 1 ? 64 : 128, dtype = (int)((s >> 9) & 3);
        const int n = sphattn_splitkv_heuristic(B, H, N, d, dtype);
        const long long tiles = ((long long)N + 63) / 64;
        if (n < 1 || n > tiles) { fprintf(stderr, "heuristic(%d,%d,%d,%d,%d) = %d\n", B, H, N, d, dtype, n); ++failures; }
    }
    EXPECT(sphattn_splitkv_heuristic(0, 1, 1, 128, 1), 1);

    // backward: aliasing matrix
    float *Z = (float*)P(0x6000000), *delta = (float*)P(0xA000000);
    void *dO = P(0x5000000), *dQ = P(0x7000000), *dK = P(0x8000000), *dV = P(0x9000000);
    EXPECT(sphattn_bwd(Q, K, V, O, dO, Z, dQ, dK, dV, delta, 1, 2, 300, 64, SPHATTN_F32, nullptr), SPHATTN_ERR_DTYPE);
    EXPECT(sphattn_bwd(Q, K, V, O, dO, Z, dQ, dK, dK, delta, 1, 2, 300, 64, SPHATTN_BF16, nullptr), SPHATTN_ERR_ALIAS);
    EXPECT(sphattn_grn_bwd(Q, K, V, (const float*)dK, O, dO, Z, dQ, dK, dV, delta, 1, 2, 1, 300, 64, SPHATTN_BF16, nullptr), SPHATTN_ERR_ALIAS);
    EXPECT(sphattn_grn_bwd(Q, K, V, nullptr, O, dO, Z, dQ, dK, dV, nullptr, 1, 2, 1, 300, 64, SPHATTN_BF16, nullptr), SPHATTN_ERR_NULL);

    // all-E4M3 forward: workspace arithmetic and checks
    const size_t need = sphattn_fp8_workspace_bytes(1, 2, 1000, 128);
    EXPECT(need, (size_t)2 * 128 * 1024 + 256);
    EXPECT(sphattn_fp8_workspace_bytes(INT_MAX, INT_MAX, INT_MAX, 128) == 0 ||
           sphattn_fp8_workspace_bytes(INT_MAX, INT_MAX, INT_MAX, 128) > need, 1);
    EXPECT(sphattn_fp8_fwd(Q, K, V, O, W, need - 1, 1, 2, 2, 1000, 128, nullptr), SPHATTN_ERR_WORKSPACE);
    EXPECT(sphattn_fp8_fwd(Q, K, V, O, K, need, 1, 2, 2, 1000, 128, nullptr), SPHATTN_ERR_ALIAS);
    EXPECT(sphattn_fp8_fwd(Q, K, V, O, W, need, 1, 2, 2, 1000, 96, nullptr), SPHATTN_ERR_HEAD_DIM);
    EXPECT(sphattn_fp8_workspace_bytes(1, 1, 130, 64), (size_t)64 * 256 + 256);
    EXPECT(sphattn_fp8_grn_fwd(Q, K, V, (const float*)O, O, W, need, 1, 2, 2, 1000, 128, nullptr), SPHATTN_ERR_ALIAS);
    EXPECT(sphattn_fp8_grn_fwd(Q, K, V, (const float*)P(0x5000001), O, W, need, 1, 2, 2, 1000, 128, nullptr), SPHATTN_ERR_ALIGN);
    EXPECT(sphattn_fp8_softmax_fwd(Q, K, V, O, W, need, 1, 3, 2, 1000, 128, nullptr), SPHATTN_ERR_SHAPE);

    for (int code = -12; code <= 1; ++code)
        if (!sphattn_strerror(code) || !sphattn_strerror(code)[0]) ++failures;
    EXPECT(sphattn_version() >= 500, 1);
    if (failures) return 1;
    puts("ok");
    return 0;
}
