// Calls the host side of every C-ABI entry point of libbra with arguments that must be refused
// before anything is enqueued (and the host-only queries with valid ones), in a build whose host
// code runs under AddressSanitizer and UndefinedBehaviorSanitizer.  No GPU is needed: no call here
// reaches a launch.  Exit status 0 means every code was as expected and no report was raised.
#include <cstdio>
#include <cstdint>
#include <climits>

#include "../../include/bra.h"

static int failures = 0;
#define EXPECT(expr, code)                                                            \
    do {                                                                              \
        const int rc_ = (expr);                                                       \
        if (rc_ != (code)) { std::printf("%s -> %d, expected %d\n", #expr, rc_, (int)(code)); ++failures; } \
    } while (0)

int main()
{
    size_t n = 0;
    void *fake = (void *)4096;
    bra_shape ok = {2, 28, 28, 64, 2, 7, 4, BRA_BF16, 0.f, BRA_PATH_AUTO};
    EXPECT(bra_workspace_bytes(&ok, &n), BRA_OK);
    EXPECT(bra_workspace_bytes(nullptr, &n), BRA_ERR_NULL);
    EXPECT(bra_workspace_bytes(&ok, nullptr), BRA_ERR_NULL);
    // every named workload and the extremes of the size checks
    const bra_shape shapes[] = {
        {1, 28, 28, 64, 2, 7, 4, BRA_F32, 0.f, BRA_PATH_AUTO},    {64, 56, 56, 64, 2, 7, 1, BRA_BF16, 0.f, BRA_PATH_AUTO},
        {64, 28, 28, 128, 4, 7, 4, BRA_BF16, 0.f, BRA_PATH_AUTO}, {64, 14, 14, 256, 8, 7, 16, BRA_BF16, 0.f, BRA_PATH_AUTO},
        {2, 128, 128, 64, 2, 8, 4, BRA_BF16, 0.f, BRA_PATH_AUTO}, {64, 7, 7, 512, 16, 7, 49, BRA_BF16, 0.f, BRA_PATH_MFMA},
        {8, 32, 32, 768, 12, 8, 12, BRA_BF16, 0.f, BRA_PATH_MFMA}, {2, 208, 304, 64, 2, 16, 4, BRA_BF16, 0.f, BRA_PATH_MFMA},
        {1, 12, 12, 48, 3, 3, 2, BRA_BF16, 0.f, BRA_PATH_GENERIC},
    };
    for (const bra_shape &s : shapes) {
        EXPECT(bra_workspace_bytes(&s, &n), BRA_OK);
        // the matrix-core backward covers heads of 32 and 64 channels, C a multiple of 64
        const bool bwd_ok = s.path != BRA_PATH_MFMA || (s.C % 64 == 0 && (s.C / s.heads == 32 || s.C / s.heads == 64));
        EXPECT(bra_backward_workspace_bytes(&s, &n), bwd_ok ? BRA_OK : BRA_ERR_UNSUPPORTED);
        EXPECT(bra_padded_workspace_bytes(&s, &n), BRA_OK);
        if (s.path != BRA_PATH_GENERIC || s.dtype == BRA_F32) EXPECT(bra_block_workspace_bytes(&s, 3 * s.C, &n), BRA_OK);
    }
    bra_shape huge = {INT32_MAX, INT32_MAX, INT32_MAX, INT32_MAX, 1, 1, 1, BRA_BF16, 0.f, BRA_PATH_AUTO};
    EXPECT(bra_workspace_bytes(&huge, &n), BRA_ERR_SHAPE);
    bra_shape big_map = {1, 8192, 8192, 64, 2, 8, 1, BRA_BF16, 0.f, BRA_PATH_MFMA};
    EXPECT(bra_workspace_bytes(&big_map, &n), BRA_ERR_UNSUPPORTED);
    bra_shape many_regions = {1, 4096, 4096, 64, 2, 2048, 1, BRA_BF16, 0.f, BRA_PATH_AUTO};
    EXPECT(bra_workspace_bytes(&many_regions, &n), BRA_ERR_SHAPE);
    bra_shape bad = ok;
    bad.S = 5;
    EXPECT(bra_workspace_bytes(&bad, &n), BRA_ERR_SHAPE);
    bad = ok; bad.k = 50;
    EXPECT(bra_workspace_bytes(&bad, &n), BRA_ERR_K);
    bad = ok; bad.dtype = 9;
    EXPECT(bra_workspace_bytes(&bad, &n), BRA_ERR_DTYPE);
    bad = ok; bad.path = -1;
    EXPECT(bra_workspace_bytes(&bad, &n), BRA_ERR_DTYPE);
    // entry points that would launch: refused on the host
    EXPECT(bra_forward(&ok, nullptr, fake, fake, fake, fake, nullptr, nullptr, fake, 1u << 30, nullptr), BRA_ERR_NULL);
    EXPECT(bra_forward(&ok, fake, fake, fake, fake, fake, nullptr, nullptr, nullptr, 1u << 30, nullptr), BRA_ERR_WORKSPACE);
    EXPECT(bra_forward(&ok, fake, fake, fake, fake, fake, nullptr, nullptr, (char *)fake + 8, 1u << 30, nullptr), BRA_ERR_WORKSPACE);
    EXPECT(bra_forward(&ok, fake, fake, fake, fake, fake, nullptr, nullptr, fake, 16, nullptr), BRA_ERR_WORKSPACE);
    EXPECT(bra_route(&ok, fake, fake, nullptr, nullptr, fake, 1u << 30, nullptr), BRA_ERR_NULL);
    EXPECT(bra_route(&ok, fake, fake, (int32_t *)fake, nullptr, fake, 16, nullptr), BRA_ERR_WORKSPACE);
    EXPECT(bra_forward_static(&ok, nullptr, fake, fake, fake, fake, nullptr, nullptr, nullptr), BRA_ERR_NULL);
    bra_shape large = {64, 28, 28, 128, 4, 7, 4, BRA_BF16, 0.f, BRA_PATH_AUTO};
    EXPECT(bra_forward_static(&large, fake, fake, fake, fake, fake, nullptr, nullptr, nullptr), BRA_ERR_TOO_LARGE);
    bra_shape odd = {1, 30, 45, 64, 2, 7, 4, BRA_BF16, 0.f, BRA_PATH_AUTO};
    EXPECT(bra_padded_workspace_bytes(&odd, &n), BRA_OK);
    EXPECT(bra_forward_padded(&odd, fake, fake, fake, fake, fake, nullptr, nullptr, nullptr, 0, nullptr), BRA_ERR_WORKSPACE);
    EXPECT(bra_backward(&ok, fake, fake, fake, fake, nullptr, fake, fake, (float *)fake, (float *)fake, (float *)fake, fake,
                        1u << 30, nullptr), BRA_ERR_NULL);
    EXPECT(bra_backward(&ok, fake, fake, fake, fake, (const int32_t *)fake, fake, fake, (float *)fake, (float *)fake,
                        (float *)fake, fake, 16, nullptr), BRA_ERR_WORKSPACE);
    EXPECT(bra_block_workspace_bytes(&ok, 0, &n), BRA_ERR_SHAPE);
    EXPECT(bra_block_forward(&ok, 192, 1e-6f, fake, nullptr, fake, nullptr, nullptr, fake, 1u << 30, nullptr), BRA_ERR_NULL);
    EXPECT(bra_profile_end(nullptr, nullptr, 4, nullptr), BRA_ERR_SHAPE);       // no session is active
    EXPECT(bra_util_copy(nullptr, fake, 16, nullptr), BRA_ERR_NULL);
    EXPECT(bra_util_copy(fake, fake, 8, nullptr), BRA_ERR_SHAPE);
    for (int code = 0; code >= -9; --code)
        if (!bra_strerror(code)) ++failures;
    if (bra_version() < 100) ++failures;
    std::printf("%d unexpected results\n", failures);
    return failures ? 1 : 0;
}
