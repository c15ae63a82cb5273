// GRPO-PODS token loss (objective of Sec. 3.2): host-side plan and the kernel families behind
// grpo_token_loss_fwd_bwd.
//
// Notation: R kept rollouts, T padded length, N = sum of lengths (valid token positions, known
// only on the device), d hidden size, V vocabulary.  Valid positions are packed into rows
// p = 0..N-1 (rollout-major; when zero-advantage rollouts are skipped, the others first); every
// kernel is launched for the worst case R*T rows and returns early for rows at or beyond N.
#pragma once

#include "common.h"

namespace pods {

struct LossArgs {
    const void* hidden;
    const void* w_lm;
    const int32_t* tokens;
    const float* old_logp;
    const float* ref_logp;   // log pi_ref(y) for the KL penalty, or null
    float kl_coef;
    const float* adv;
    const int32_t* lengths;
    int32_t R, T, d, V;
    pods_dtype dt;
    float clip_eps, grad_scale;
    float* loss;
    float* logp_out;
    float* d_hidden;
    float* d_w_lm;
    bool accumulate_d_w;   // d_w_lm += gradient instead of d_w_lm = gradient
    bool skip_zero_adv;    // rollouts with a_i == 0 take no part in the backward pass
    unsigned char* workspace;
    size_t workspace_bytes;
    hipStream_t stream;
};

// Device header at the start of the workspace.
struct LossHeader {
    int32_t n_valid;     // N
    uint32_t gmax_bits;  // bit pattern of max_t |g_t| (non-negative floats order as integers)
    int32_t n_bwd;       // packed rows the backward pass covers: N, or only the rows of rollouts with
                         // a non-zero advantage (they are packed first when those are skipped)
    int32_t pad[61];
};

// Scale 2^-floor(log2 gmax) that brings the per-token weights g_t into [0, 2).
__device__ __forceinline__ float g_range_scale(const LossHeader* hdr) {
    const uint32_t e = (hdr->gmax_bits >> 23) & 0xFFu;
    if (hdr->gmax_bits == 0u) return 1.0f;
    const uint32_t se = e == 0u ? 253u : (e >= 253u ? 1u : 254u - e);
    return __uint_as_float(se << 23);
}

// Fixed power-of-two scales of the fp16 operands of the two gradient contractions.
constexpr float kQScale = 16384.0f;  // q = kQScale softmax (0 at v = y): 0 <= q <= 2^14
constexpr float kWScale = 256.0f;    // the fp16 weight copy of the gradient contractions holds kWScale * W

constexpr int kTile = 256;          // token / vocab / hidden tile edge of the matrix-core kernels
constexpr int kDefaultVocabChunk = 8192;

struct LossPlan {
    int64_t ncap;     // R*T
    int64_t ncap_ld;  // ncap rounded up to kTile: rows of the per-token arrays
    bool mfma;        // bf16 inputs with d % 64 == 0 take the matrix-core path
    int slots;        // forward partial slots per token
    int vc;           // vocabulary chunk of the backward pass (multiple of kTile); 0 on the plain path
    int nchunks;
    int64_t ldq;      // row pitch of q in elements: vc plus one tile, so rows do not sit a power of two apart
    int64_t vld;      // rows of the fp16 weight copy = nchunks * vc (zero past V)
    int64_t vld_t;    // columns of the transposed fp16 weight copy = V rounded up to kTile
    int loss_blocks;
    size_t off_hdr, off_offsets, off_rowmap, off_tok, off_lse, off_zy, off_g, off_coef, off_pmax, off_psum,
        off_losspart, off_wtt, off_htt, off_wt, off_ht, off_dz, total;
};

// mode 0: recommended size; mode 1: minimum size; otherwise `mode` is the number of bytes
// available and the largest vocabulary chunk that fits is chosen.
LossPlan plan_loss(int32_t R, int32_t T, int32_t d, int32_t V, pods_dtype dt, size_t mode);

pods_status run_loss(const LossArgs& a);

// Plain kernels (fp32 arithmetic, any shape): loss_simple.hip
pods_status simple_forward(const LossArgs& a, const LossPlan& p);
pods_status simple_backward(const LossArgs& a, const LossPlan& p);

// Matrix-core kernels (bf16 inputs): loss_mfma.hip
pods_status mfma_forward(const LossArgs& a, const LossPlan& p);
pods_status mfma_backward(const LossArgs& a, const LossPlan& p);

}  // namespace pods
