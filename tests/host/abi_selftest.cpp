// Host-only self test of the C ABI's argument handling, meant to be built with the host pass under
// -fsanitize=address,undefined and linked against stub launchers (no GPU code runs): every entry point is
// called with bad and with empty arguments and must answer with the documented status code.
#include <cstdint>
#include <cstdio>

#include "hyena.h"

int main() {
    char* const base = reinterpret_cast<char*>(0x100000);
    void* P[12];
    for (int i = 0; i < 12; ++i) P[i] = base + 0x100000 * i;
    const float* H[4] = {reinterpret_cast<const float*>(base + 0x4000000), reinterpret_cast<const float*>(base + 0x4100000),
                         reinterpret_cast<const float*>(base + 0x4200000), reinterpret_cast<const float*>(base + 0x4300000)};
    float* DH = reinterpret_cast<float*>(base + 0x4400000);
    int bad = 0;
#define EXPECT(call, code) do { if ((call) != (code)) { std::printf("line %d: unexpected status\n", __LINE__); ++bad; } } while (0)
    EXPECT(hyena_se_fwd(nullptr, P[1], P[2], H[0], P[3], 1, 8, 16, 3, 1, HY_F32, nullptr), HY_ERR_NULL);
    EXPECT(hyena_se_fwd(P[0], P[1], P[2], H[0], P[3], 1, 8, 16, 0, 1, HY_F32, nullptr), HY_ERR_SHAPE);
    EXPECT(hyena_se_fwd(P[0], P[1], P[2], H[0], P[3], 1, 8, 16, 3, 5, HY_F32, nullptr), HY_ERR_SHAPE);
    EXPECT(hyena_se_fwd(P[0], P[1], P[2], H[0], P[3], 1, 8, 16, 3, 1, 9, nullptr), HY_ERR_DTYPE);
    EXPECT(hyena_se_fwd(P[0], P[1], P[2], H[0], P[1], 1, 8, 16, 3, 1, HY_BF16, nullptr), HY_ERR_ALIGN);
    EXPECT(hyena_se_fwd(P[0], P[1], P[2], H[0], P[3], INT64_MAX / 2, 8, 16, 3, 1, HY_BF16, nullptr), HY_ERR_SHAPE);
    EXPECT(hyena_se_fwd(P[0], P[1], P[2], H[0], P[3], 0, 8, 16, 3, 1, HY_BF16, nullptr), HY_OK);
    EXPECT(hyena_se_fwd(P[0], P[1], P[2], H[0], P[3], 1, 8, 16, 3, 1, HY_BF16, nullptr), HY_OK);
    EXPECT(hyena_mr_fwd(P[0], P[1], P[2], H[0], P[3], 1, 8, 64, 128, 16, HY_BF16, nullptr), HY_OK);
    EXPECT(hyena_mr_fwd(P[0], P[1], P[2], H[0], static_cast<char*>(P[3]) + 2, 1, 8, 64, 128, 16, HY_BF16, nullptr), HY_ERR_ALIGN);
    EXPECT(hyena_featurize_fwd(P[0], H[0], P[1], 1, 8, 16, 7, 1, HY_F32, nullptr), HY_OK);
    EXPECT(hyena_featurize_fwd(P[0], nullptr, P[1], 1, 8, 16, 7, 1, HY_F32, nullptr), HY_ERR_NULL);
    EXPECT(hyena_featurize3_fwd(P[0], P[1], P[2], H[0], H[1], H[2], P[3], P[4], P[3], 1, 8, 16, 7, 1, HY_F32, nullptr), HY_ERR_ALIGN);
    EXPECT(hyena_featurize3_fwd(P[0], P[1], P[2], H[0], H[1], H[2], P[3], P[4], P[5], 1, 8, 16, 7, 1, HY_F32, nullptr), HY_OK);
    EXPECT(hyena_chain_fwd(P[0], P[1], P[2], H[0], H[1], H[2], H[3], P[3], nullptr, 0, 1, 8, 128, 7, 1, 128, 16, HY_BF16, nullptr), HY_OK);
    EXPECT(hyena_chain_fwd(P[0], P[1], P[2], H[0], H[1], H[2], H[3], P[3], nullptr, 0, 1, 8, 128, 7, 1, 128, 16, HY_F32, nullptr), HY_ERR_NULL);
    EXPECT(hyena_chain_fwd(P[0], P[1], P[2], H[0], H[1], H[2], H[3], P[3], P[6], 3 * 8 * 128 * 4, 1, 8, 128, 7, 1, 128, 16, HY_F32, nullptr), HY_OK);
    EXPECT(hyena_chain_fwd(P[0], P[1], P[2], H[0], H[1], H[2], H[3], P[3], P[6], 3 * 8 * 128 * 4 - 1, 1, 8, 128, 7, 1, 128, 16, HY_F32, nullptr), HY_ERR_SHAPE);
    EXPECT(hyena_chain_fwd(P[0], P[1], P[2], H[0], H[1], H[2], reinterpret_cast<const float*>(P[3]), P[3], P[6], 1 << 20, 1, 8, 128, 7, 1, 128, 16, HY_F32, nullptr), HY_ERR_ALIGN);
    EXPECT(hyena_chain_fwd(P[0], P[1], P[2], H[0], H[1], H[2], H[3], P[3], P[2], 1 << 20, 1, 8, 128, 7, 1, 128, 16, HY_F32, nullptr), HY_ERR_ALIGN);
    if (hyena_chain_workspace_bytes(1, 8, 128, 7, 1, 128, 16, HY_F32) != 3 * 8 * 128 * 4) ++bad;
    if (hyena_chain_workspace_bytes(1, 8, 128, 7, 1, 128, 16, HY_BF16) != 0) ++bad;
    EXPECT(hyena_se_bwd(P[0], P[1], P[2], P[3], H[0], P[4], P[5], P[6], DH, P[7], 1 << 16, 1, 8, 16, 3, 1, HY_BF16, nullptr), HY_OK);
    EXPECT(hyena_se_bwd(P[0], P[1], P[2], P[3], H[0], P[4], P[5], P[6], DH, P[7], 8, 1, 8, 16, 3, 1, HY_BF16, nullptr), HY_ERR_SHAPE);
    EXPECT(hyena_se_bwd(P[0], P[1], P[2], P[3], H[0], P[4], P[5], P[6], DH, nullptr, 0, 1, 8, 16, 3, 1, HY_BF16, nullptr), HY_ERR_NULL);
    EXPECT(hyena_mr_bwd(P[0], P[1], P[2], P[3], H[0], P[4], P[5], P[6], DH, nullptr, 0, 1, 8, 40, 50, 1, HY_BF16, nullptr), HY_OK);
    EXPECT(hyena_mr_bwd(P[0], P[1], P[2], P[3], H[0], P[4], P[5], P[4], DH, nullptr, 0, 1, 8, 40, 50, 1, HY_BF16, nullptr), HY_ERR_ALIGN);
    EXPECT(hyena_mr_bwd(P[0], P[1], P[2], P[3], H[0], P[4], P[5], P[6], DH, nullptr, 0, 0, 8, 40, 50, 1, HY_BF16, nullptr), HY_OK);
    if (hyena_bwd_workspace_bytes(1, 8, 16, 3, 1, HY_BF16) != 16 * 3 * 4) ++bad;
    // a filter table or the filter gradient inside a written activation
    EXPECT(hyena_se_fwd(P[0], P[1], P[2], reinterpret_cast<const float*>(P[3]), P[3], 1, 8, 16, 3, 1, HY_BF16, nullptr), HY_ERR_ALIGN);
    EXPECT(hyena_se_bwd(P[0], P[1], P[2], P[3], H[0], P[4], P[5], P[6], reinterpret_cast<float*>(P[5]), P[7], 1 << 16, 1, 8, 16, 3, 1, HY_BF16, nullptr), HY_ERR_ALIGN);
    // Hyena-LI with the library's own scratch: same checks, no workspace argument; a scan that needs more than the
    // static buffer is refused before anything is launched
    EXPECT(hyena_li_fwd_static(P[0], P[1], P[2], H[0], H[1], P[3], 1, 8, 64, 16, 16, HY_BF16, nullptr), HY_OK);
    EXPECT(hyena_li_fwd_static(P[0], P[1], P[2], H[0], nullptr, P[3], 1, 8, 64, 16, 16, HY_BF16, nullptr), HY_ERR_NULL);
    EXPECT(hyena_li_fwd_static(P[0], P[1], P[2], H[0], H[1], P[3], 1, 8, 64, 65, 16, HY_BF16, nullptr), HY_ERR_UNSUPPORTED);
    EXPECT(hyena_li_fwd_static(P[0], P[1], P[2], H[0], H[1], P[3], 1, 8, 64, 16, 16, HY_F32, nullptr), HY_OK);
    {
        char* const far = reinterpret_cast<char*>(1ull << 40);  // 128 MiB tensors, 4 GiB apart
        EXPECT(hyena_li_fwd_static(far, far + (1ull << 32), far + (2ull << 32), H[0], H[1], far + (3ull << 32), 1, 1 << 14,
                                   4096, 16, 16, HY_BF16, nullptr), HY_ERR_SCRATCH);
    }
    EXPECT(hyena_stream_copy(P[0], P[1], 24, nullptr), HY_ERR_SHAPE);
    EXPECT(hyena_stream_copy(P[0], P[1], 64, nullptr), HY_OK);
    EXPECT(hyena_set_option("se_vec", 3), HY_ERR_SHAPE);
    EXPECT(hyena_set_option("nope", 1), HY_ERR_UNSUPPORTED);
    EXPECT(hyena_set_option(nullptr, 1), HY_ERR_NULL);
    for (int s = 0; s < 9; ++s)
        if (!hyena_status_string(s)) ++bad;
    std::printf("abi selftest: %d problem(s), version %d\n", bad, hyena_version());
    return bad != 0;
}
