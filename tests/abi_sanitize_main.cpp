// Drives the host side of the C ABI (argument validation and the workspace planning, none of which touches a
// device) in a build whose host code is compiled with AddressSanitizer and UndefinedBehaviorSanitizer.
#include <cstdint>
#include <cstdio>
#include <cstring>

#include "pods.h"

#define EXPECT(call, want)                                                              \
    do {                                                                                \
        const int got_ = (int)(call);                                                   \
        if (got_ != (int)(want)) {                                                      \
            std::fprintf(stderr, "%s: got %d, want %d (%s)\n", #call, got_, (int)(want), pods_last_error()); \
            return 1;                                                                   \
        }                                                                               \
    } while (0)

int main() {
    void* one = reinterpret_cast<void*>(256);   // never dereferenced: every call below fails validation first
    float* f = static_cast<float*>(one);
    int32_t* i = static_cast<int32_t*>(one);
    EXPECT(pods_select(nullptr, 1, 4, 2, i, nullptr, nullptr), PODS_ERR_INVALID_ARG);
    EXPECT(pods_select(f, 1, 4, 5, i, nullptr, nullptr), PODS_ERR_INVALID_ARG);
    EXPECT(pods_select(f, 0, 4, 2, i, nullptr, nullptr), PODS_ERR_INVALID_ARG);
    EXPECT(pods_select(f, 1, 5000, 2, i, nullptr, nullptr), PODS_ERR_UNSUPPORTED);
    EXPECT(pods_downsample(f, nullptr, 1, 4, 2, PODS_RULE_RAND, i, nullptr, nullptr), PODS_ERR_INVALID_ARG);
    EXPECT(pods_downsample(f, nullptr, 1, 4, 2, (pods_rule)9, i, nullptr, nullptr), PODS_ERR_INVALID_ARG);
    EXPECT(pods_advantage(f, nullptr, 1, 4, 2, 0.0f, f, nullptr), PODS_ERR_INVALID_ARG);
    EXPECT(pods_advantage(f, i, 1, 4, 2, -1.0f, f, nullptr), PODS_ERR_INVALID_ARG);
    EXPECT(pods_check_rewards(f, 1, 4, nullptr, nullptr), PODS_ERR_INVALID_ARG);
    EXPECT(pods_gather_rows(one, i, 1, 4, 2, 0, one, nullptr), PODS_ERR_INVALID_ARG);
    pods_record rec[PODS_MAX_RECORDS + 1];
    std::memset(rec, 0, sizeof(rec));
    EXPECT(pods_downsample_gather(f, nullptr, 1, 4, 2, PODS_RULE_MAXVAR, 0.0f, 0, rec, PODS_MAX_RECORDS + 1, i, nullptr, f,
                                  nullptr), PODS_ERR_INVALID_ARG);
    EXPECT(pods_downsample_gather(f, nullptr, 1, 4, 2, PODS_RULE_MAXVAR, 0.0f, 0, rec, 2, i, nullptr, f, nullptr),
           PODS_ERR_INVALID_ARG);   // records with null pointers
    EXPECT(grpo_token_loss_fwd_bwd(nullptr, one, i, f, f, nullptr, 2, 8, 64, 100, PODS_BF16, 0.2f, 1.0f, f, nullptr, f, f,
                                   one, 1 << 20, nullptr), PODS_ERR_INVALID_ARG);
    EXPECT(grpo_token_loss_fwd_bwd(one, one, i, f, f, nullptr, 2, 8, 64, 100, PODS_BF16, -0.2f, 1.0f, f, nullptr, f, f,
                                   one, 1 << 20, nullptr), PODS_ERR_INVALID_ARG);
    EXPECT(grpo_token_loss_fwd_bwd(one, one, i, f, f, nullptr, 2, 8, 20000, 100, PODS_BF16, 0.2f, 1.0f, f, nullptr, f, f,
                                   one, 1 << 20, nullptr), PODS_ERR_UNSUPPORTED);
    EXPECT(grpo_token_loss_fwd_bwd(one, one, i, f, f, nullptr, 2, 8, 64, 100, PODS_BF16, 0.2f, 1.0f, f, nullptr, f, f,
                                   one, 16, nullptr), PODS_ERR_WORKSPACE);
    EXPECT(grpo_token_loss_fwd_bwd(one, one, i, f, f, nullptr, 2, 8, 64, 100, PODS_BF16, 0.2f, 1.0f, f, nullptr, f, f,
                                   reinterpret_cast<void*>(264), 1 << 20, nullptr), PODS_ERR_WORKSPACE);
    EXPECT(grpo_token_loss_fwd_bwd_ex(one, one, i, f, nullptr, f, nullptr, 2, 8, 64, 100, PODS_BF16, 0.2f, 0.1f, 1.0f, 0, f,
                                      nullptr, f, f, one, 1 << 20, nullptr), PODS_ERR_INVALID_ARG);   // kl without ref
    EXPECT(grpo_token_loss_fwd_bwd_ex(one, one, i, f, nullptr, f, nullptr, 2, 8, 64, 100, PODS_BF16, 0.2f, 0.0f, 1.0f, 64, f,
                                      nullptr, f, f, one, 1 << 20, nullptr), PODS_ERR_INVALID_ARG);   // unknown flag
    EXPECT(grpo_token_loss_fwd_bwd_static(one, one, i, f, f, nullptr, 512, 1024, 2048, 151936, PODS_BF16, 0.2f, 1.0f, f,
                                          nullptr, f, f, nullptr), PODS_ERR_UNSUPPORTED);
    EXPECT(grpo_token_loss_report(one, nullptr, nullptr), PODS_ERR_INVALID_ARG);
    // workspace planning: host arithmetic only
    const int shapes[][4] = {{2, 64, 4096, 151936}, {512, 1024, 2048, 151936}, {3, 50, 128, 1000}, {1, 1, 64, 5},
                             {128, 2048, 3584, 152064}, {16, 64, 256, 1024}};
    for (const auto& s : shapes) {
        for (int dt = 0; dt < 2; ++dt) {
            const size_t least = grpo_token_loss_workspace_min_bytes(s[0], s[1], s[2], s[3], (pods_dtype)dt);
            const size_t rec_b = grpo_token_loss_workspace_bytes(s[0], s[1], s[2], s[3], (pods_dtype)dt);
            if (least == 0 || least > rec_b) return 2;
            for (size_t b = least; b <= rec_b + (8u << 20); b += (rec_b - least) / 37 + 4096) {
                const size_t used = grpo_token_loss_workspace_used_bytes(s[0], s[1], s[2], s[3], (pods_dtype)dt, b);
                if (used < least || used > b) return 3;
            }
        }
    }
    if (grpo_token_loss_workspace_bytes(0, 1, 1, 1, PODS_F32) != 0) return 4;
    std::printf("abi sanitizer run ok\n");
    return 0;
}
