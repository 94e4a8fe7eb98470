// Host-side exercise of libflurka's validation, sizing arithmetic and stage timer, meant to be built and
// linked with -fsanitize=address,undefined against a host-instrumented build of the library
// (paper_2306_15799_amd/build.py: build_sanitized).  Needs no GPU: every call here returns before any launch.
// Exit code 0 = every expectation held (the sanitizers abort the process on a finding).
#include <stdio.h>
#include <stdlib.h>
#include <vector>

#include "flurka.h"

static int failures = 0;
#define EXPECT(cond)                                                   \
    do {                                                               \
        if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } \
    } while (0)

int main() {
    void* fake = (void*)0x7F0000000000;       // aligned, never dereferenced: validation fails first
    // sizes at the accepted limits: size_t arithmetic must not wrap
    const size_t c_big = flurka_ctx_bytes(1, FLURKA_MAX_BATCH_HEADS, FLURKA_MAX_SEQ, FLURKA_MAX_FEATURE_DIM,
                                          FLURKA_MAX_SEQ, FLURKA_MAX_FEATURE_DIM, FLURKA_F32, FLURKA_PHI_PERFORMER);
    EXPECT(c_big > (size_t)FLURKA_MAX_BATCH_HEADS * FLURKA_MAX_SEQ * FLURKA_MAX_FEATURE_DIM);
    for (int pass = 0; pass < 2; ++pass)
        for (int algo = 0; algo < 3; ++algo) {
            const size_t w = flurka_workspace_bytes(1, FLURKA_MAX_BATCH_HEADS, FLURKA_MAX_SEQ, FLURKA_MAX_FEATURE_DIM,
                                                    FLURKA_MAX_SEQ, FLURKA_MAX_FEATURE_DIM, FLURKA_F32,
                                                    FLURKA_PHI_PERFORMER, (flurka_pass)pass, (flurka_algo)algo);
            EXPECT(algo == FLURKA_ALGO_FAST ? w == 0 : w > 0);
        }
    EXPECT(flurka_ctx_bytes(1, FLURKA_MAX_BATCH_HEADS + 1, 8, 8, 8, 8, FLURKA_F32, FLURKA_PHI_PERFORMER) == 0);
    size_t offs[6];
    EXPECT(flurka_ctx_layout(1, 1, 512, 64, 64, 64, FLURKA_F32, FLURKA_PHI_PERFORMER, offs) == FLURKA_OK);
    EXPECT(offs[5] == 12416);
    // a sweep of shapes through every sizing helper (MFMA path included: bf16, tile multiples)
    const int ns[] = {64, 192, 4096, 65536}, ks[] = {1, 100, 512, 1 << 18}, ms[] = {32, 96, 256, 512};
    for (int d : {64, 128})
        for (int n : ns)
            for (int k : ks)
                for (int m : ms)
                    for (int bh : {1, 5, 64}) {
                        for (int pass = 0; pass < 2; ++pass) {
                            const int sup = flurka_fast_path_supported(1, bh, n, d, k, m, FLURKA_BF16, FLURKA_PHI_PERFORMER, (flurka_pass)pass);
                            const size_t w = flurka_workspace_bytes(1, bh, n, d, k, m, FLURKA_BF16, FLURKA_PHI_PERFORMER,
                                                                    (flurka_pass)pass, FLURKA_ALGO_FAST);
                            EXPECT((sup != 0) == (w != 0));
                        }
                        (void)flurka_fused_w_supported(1, bh, n, d, k, m, 64 * bh, FLURKA_BF16, FLURKA_PHI_PERFORMER);
                        (void)flurka_fused_w_workspace_bytes(1, bh, n, d, k, m, 64 * bh, FLURKA_BF16, FLURKA_PHI_PERFORMER);
                    }
    // validation order of the three forward entry points and the backward
    EXPECT(flurka_attn_fwd(nullptr, fake, fake, fake, fake, fake, fake, fake, 1 << 30, fake, 1 << 30, 1, 1, 512, 64, 64, 64, 1,
                           FLURKA_F32, FLURKA_PHI_PERFORMER, FLURKA_ALGO_GENERIC, nullptr) == FLURKA_ERR_NULL);
    EXPECT(flurka_attn_fwd(fake, fake, fake, fake, fake, fake, fake, fake, 16, fake, 1 << 30, 1, 1, 512, 64, 64, 64, 1,
                           FLURKA_F32, FLURKA_PHI_PERFORMER, FLURKA_ALGO_GENERIC, nullptr) == FLURKA_ERR_WORKSPACE);
    EXPECT(flurka_attn_fwd_static(fake, fake, fake, fake, fake, fake, fake, fake, 16, 1, 1, 512, 64, 64, 64, 1,
                                  FLURKA_F32, FLURKA_PHI_PERFORMER, FLURKA_ALGO_GENERIC, nullptr) == FLURKA_ERR_WORKSPACE);
    EXPECT(flurka_attn_fwd_fused_w(fake, fake, fake, fake, fake, fake, fake, fake, fake, fake, 1 << 30, fake, 16, 1, 4, 512,
                                   64, 64, 64, 256, 1, FLURKA_BF16, FLURKA_PHI_PERFORMER, nullptr) == FLURKA_ERR_WORKSPACE);
    EXPECT(flurka_attn_bwd(fake, fake, fake, fake, fake, fake, fake, fake, fake, 1 << 30, fake, fake, fake, fake, fake, fake,
                           16, 1, 1, 512, 64, 64, 64, 1, FLURKA_F32, FLURKA_PHI_PERFORMER, FLURKA_ALGO_GENERIC,
                           nullptr) == FLURKA_ERR_WORKSPACE);
    {   // extended entry points: options are read before anything is launched
        flurka_options opt = {1, 1, fake};
        EXPECT(flurka_attn_bwd_ex(fake, fake, fake, fake, fake, fake, fake, fake, fake, 1 << 30, fake, fake, fake, fake, fake,
                                  fake, 16, 1, 2, 512, 64, 64, 64, 1, FLURKA_BF16, FLURKA_PHI_PERFORMER, FLURKA_ALGO_AUTO,
                                  &opt, nullptr) == FLURKA_ERR_WORKSPACE);
        EXPECT(flurka_attn_fwd_ex(fake, fake, fake, fake, fake, fake, fake, fake, 1 << 30, fake, 16, 1, 2, 512, 64, 64, 64, 1,
                                  FLURKA_BF16, FLURKA_PHI_PERFORMER, FLURKA_ALGO_FAST, &opt, nullptr) == FLURKA_ERR_UNSUPPORTED);
        EXPECT(flurka_baseline_fwd(FLURKA_BASELINE_LINFORMER, fake, fake, fake, fake, fake, nullptr, fake, fake, 16, fake,
                                   1 << 30, 1, 2, 512, 64, 64, 64, 1, FLURKA_BF16, FLURKA_PHI_PERFORMER,
                                   nullptr) == FLURKA_ERR_WORKSPACE);
    }
    // stage timer: read while disabled, enable/disable cycles (without a GPU enabling fails cleanly)
    std::vector<int> ids(8);
    std::vector<float> ms_(8);
    EXPECT(flurka_profile_read(ids.data(), ms_.data(), 8) == 0);
    for (int i = 0; i < 3; ++i) {
        const flurka_status st = flurka_profile_enable(1);
        EXPECT(st == FLURKA_OK || st == FLURKA_ERR_LAUNCH);
        EXPECT(flurka_profile_read(ids.data(), ms_.data(), 8) == 0);
        EXPECT(flurka_profile_read(nullptr, ms_.data(), 8) == 0);
        EXPECT(flurka_profile_enable(0) == FLURKA_OK);
    }
    for (int i = -1; i < 30; ++i) EXPECT(flurka_profile_stage_name(i) != nullptr);
    for (int i = 0; i < 8; ++i) EXPECT(flurka_status_str((flurka_status)i) != nullptr);
    printf(failures ? "%d expectation(s) failed\n" : "all expectations held\n", failures);
    return failures ? 1 : 0;
}
